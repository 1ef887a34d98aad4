"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds NO arithmetic of the method: it only draws random numbers
and states layer shapes.  The same arrays are handed to the CPU oracle and to
the GPU library by the tests and the benchmark.

The paper measures on MNIST (Sec. 6.2) and CIFAR-10 (Sec. 6.3) with weights
trained by BinaryNet, and on two dense 8192 x 8192 matrices (Sec. 6.1).  None of
those datasets or weights is used here: the arrays below have the same shapes
and value domains (+-1 weights and activations, real-valued images in [0,1)),
drawn i.i.d. from ``numpy.random.default_rng(SEED0 + config number)``.
"""
from __future__ import annotations

import numpy as np

SEED0 = 170507175
BN_EPS = 1e-4

# Sec. 6.2: the MNIST multi-layer perceptron (784-4096-4096-4096-10).
MLP_SIZES = (784, 4096, 4096, 4096, 10)

# Sec. 6.3: the CIFAR-10 VGG-like network.  ("conv", C_in, C_out) are 3x3,
# stride 1, pad 1; ("pool",) is 2x2 stride 2; ("dense", K, N).
CNN_LAYERS = (
    ("conv", 3, 128),
    ("conv", 128, 128),
    ("pool",),
    ("conv", 128, 256),
    ("conv", 256, 256),
    ("pool",),
    ("conv", 256, 512),
    ("conv", 512, 512),
    ("pool",),
    ("dense", 8192, 1024),
    ("dense", 1024, 1024),
    ("dense", 1024, 10),
)


def rng_for(config: int, stream: int = 0) -> np.random.Generator:
    """Generator for workload configuration ``config`` (1-5); ``stream`` picks an independent sub-stream."""
    return np.random.default_rng([SEED0 + int(config), int(stream)])


def pm1(rng: np.random.Generator, shape) -> np.ndarray:
    """+-1 values, i.i.d. with probability one half, as int8."""
    return (rng.integers(0, 2, size=shape, dtype=np.int8) * 2 - 1).astype(np.int8)


def bn_params(rng: np.random.Generator, channels: int):
    """(gamma, beta, mean, var): gamma, beta, mean ~ N(0,1); var ~ U(0.5, 2); float32."""
    gamma = rng.standard_normal(channels).astype(np.float32)
    beta = rng.standard_normal(channels).astype(np.float32)
    mean = rng.standard_normal(channels).astype(np.float32)
    var = rng.uniform(0.5, 2.0, channels).astype(np.float32)
    return gamma, beta, mean, var


def config1(m: int = 64, n: int = 1024, k: int = 1024):
    """One binary dense layer: activations A [m][k] and weights B [n][k], +-1."""
    r = rng_for(1)
    return pm1(r, (m, k)), pm1(r, (n, k))


def config2(batch: int = 32, h: int = 32, w: int = 32, c: int = 128, l2: int = 128):
    """One binary conv layer: x NHWC +-1, 3x3 filters [l2][3][3][c] +-1, BN per output channel."""
    r = rng_for(2)
    x = pm1(r, (batch, h, w, c))
    f = pm1(r, (l2, 3, 3, c))
    return x, f, bn_params(r, l2)


def mlp_params(sizes=MLP_SIZES):
    """Weights [N][K] +-1 per layer and BN parameters after every layer but the last."""
    r = rng_for(3, 1)
    layers = []
    for i in range(len(sizes) - 1):
        k, n = sizes[i], sizes[i + 1]
        w = pm1(r, (n, k))
        bnp = bn_params(r, n) if i < len(sizes) - 2 else None
        layers.append({"w": w, "bn": bnp})
    return layers


def mlp_input(batch: int, k: int = MLP_SIZES[0]) -> np.ndarray:
    """Real-valued inputs in [0,1), float32 [batch][k]."""
    return rng_for(3, 0).random((batch, k), dtype=np.float32)


def cnn_params(layers=CNN_LAYERS):
    """Filters [L2][3][3][C] / dense weights [N][K], +-1, with BN after every layer but the last."""
    r = rng_for(4, 1)
    out = []
    last = max(i for i, l in enumerate(layers) if l[0] != "pool")
    for i, l in enumerate(layers):
        if l[0] == "pool":
            out.append({"kind": "pool"})
            continue
        if l[0] == "conv":
            w = pm1(r, (l[2], 3, 3, l[1]))
        else:
            w = pm1(r, (l[2], l[1]))
        bnp = bn_params(r, l[2]) if i != last else None
        out.append({"kind": l[0], "w": w, "bn": bnp})
    return out


def cnn_input(batch: int, h: int = 32, w: int = 32, c: int = 3) -> np.ndarray:
    """Real-valued images in [0,1), float32 NHWC."""
    return rng_for(4, 0).random((batch, h, w, c), dtype=np.float32)


def config5_square(n: int):
    """Two +-1 matrices [n][n] for the square binary-GEMM sweep."""
    r = rng_for(5, n)
    return pm1(r, (n, n)), pm1(r, (n, n))


def config5_gemv(k: int = 16384, n: int = 16384):
    """A +-1 vector [1][k] and a +-1 matrix [n][k] for the batch-1 product."""
    r = rng_for(5, 1)
    return pm1(r, (1, k)), pm1(r, (n, k))
