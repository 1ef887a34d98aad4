"""Whole-network oracle forwards -- TEST INFRASTRUCTURE (see ``oracle/__init__.py``).

The two networks of the paper's evaluation, written as a plain chain of the
oracle's layer definitions on unpacked +-1 values:

* Sec. 6.2: the MNIST multi-layer perceptron, a real-valued first dense layer
  followed by binary dense layers;
* Sec. 6.3: the CIFAR-10 VGG-like network, a real-valued first convolution,
  binary 3x3 convolutions (border treated as -1, Sec. 5.2 "Zero-padding for
  convolutions"), 2x2 max-pooling and binary dense layers.

Batch-norm then sign (Eq. 1) follows every layer but the last, which returns
raw int32 scores.  Pooling acts on the +-1 activations after the sign.

Each forward returns a list with one record per layer holding the
pre-activation (``pre``), the batch-norm output (``y``, float64) and the +-1
activation (``act``).  ``first_act`` lets a caller substitute the first layer's
activation, so that the binary layers can be checked exactly from a given
starting point.
"""
from __future__ import annotations

import numpy as np

from . import bn, conv_f64, conv_pm1, dense_f64, dense_pm1, dense_u8, maxpool_pm1, sign


def _bn_sign(pre, bnp, eps):
    y = bn(pre, *bnp, eps)
    return y, sign(y)


def mlp_forward(x: np.ndarray, layers, eps: float, first_act: np.ndarray | None = None):
    """Sec. 6.2 network.  ``x`` float32 [B][784]; ``layers`` = [{"w": int8 [N][K], "bn": ...}]."""
    trace = []
    act = None
    for i, layer in enumerate(layers):
        if i == 0:
            # real-valued input (float first layer) or 8-bit fixed-precision input (Sec. 4.3:
            # the exact integer product that the bit-plane evaluation of Eq. 3 reproduces)
            pre = dense_u8(x, layer["w"]) if x.dtype == np.uint8 else dense_f64(x, layer["w"])
        else:
            pre = dense_pm1(act, layer["w"])
        rec = {"pre": pre}
        if layer["bn"] is not None:
            rec["y"], rec["act"] = _bn_sign(pre, layer["bn"], eps)
            if i == 0 and first_act is not None:
                rec["act"] = np.ascontiguousarray(first_act, dtype=np.int8)
            act = rec["act"]
        trace.append(rec)
    return trace


def cnn_forward(x: np.ndarray, layers, eps: float, first_act: np.ndarray | None = None,
                pad_value: int = -1):
    """Sec. 6.3 network.  ``x`` float32 NHWC [B][32][32][3]; ``layers`` as from the generator:
    {"kind": "conv"|"dense"|"pool", "w": ..., "bn": ...}.  ``pad_value`` is the border value of
    the binary convolutions: -1 (the uncorrected kernel of Sec. 5.2 "Zero-padding for
    convolutions") or 0 (true zero padding, what the correction matrix restores)."""
    trace = []
    act = None
    for i, layer in enumerate(layers):
        kind = layer["kind"]
        if kind == "pool":
            act = maxpool_pm1(act, 2, 2)
            trace.append({"act": act})
            continue
        if kind == "conv":
            if i == 0:
                pre = conv_f64(x, layer["w"], stride=1, pad=1)
            else:
                pre = conv_pm1(act, layer["w"], stride=1, pad=1, pad_value=pad_value)
        else:
            if act.ndim == 4:
                # Flatten [B][H][W][C] in storage order (Sec. 5.1: element (m,n,l) at (m*N+n)*L+l).
                act = act.reshape(act.shape[0], -1)
            pre = dense_pm1(act, layer["w"])
        rec = {"pre": pre}
        if layer["bn"] is not None:
            rec["y"], rec["act"] = _bn_sign(pre, layer["bn"], eps)
            if i == 0 and first_act is not None:
                rec["act"] = np.ascontiguousarray(first_act, dtype=np.int8)
            act = rec["act"]
        trace.append(rec)
    return trace
