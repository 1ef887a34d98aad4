"""Host-side drivers that chain the library calls into the two networks of the paper's
evaluation (arXiv 1705.07175): the MNIST multi-layer perceptron of Sec. 6.2 and the
CIFAR-10 VGG-like network of Sec. 6.3.

Following the paper, weights are bit-packed once when the network is built (Sec. 6.2
"Binary optimized layers"), batch-norm is folded to integer thresholds at the same
time, and every activation / workspace buffer is allocated up front (Sec. 3
"Technical highlights"): ``forward`` only enqueues kernels on the current stream, so
it can be captured in a HIP graph.  The first layer is real-valued (fp32), all others
are binary; the last layer returns raw int32 scores.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as esp


def _dev_f32(a, device):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


class _FoldedBN:
    """Batch-norm + sign folded at load time: integer thresholds + flip bits for the binary
    layers, float thresholds + signs for the real-valued first layer."""

    def __init__(self, bnp, eps, device, integer=True):
        if integer:
            thr, flip = esp.bn_fold(*bnp, float(eps))
            self.thr = torch.from_numpy(thr).to(device)
            self.flip = esp.to_packed_tensor(flip, device)
        else:
            thr, sgn = esp.bn_fold_f32(*bnp, float(eps))
            self.thr = torch.from_numpy(thr).to(device)
            self.sgn = torch.from_numpy(sgn).to(device)


def _pack_weights(w_pm1: np.ndarray, device) -> torch.Tensor:
    """+-1 weights [N][...][K] -> packed words via the library's own pack kernel."""
    return esp.pack_f32(_dev_f32(w_pm1, device))


class BinaryMLP:
    """Sec. 6.2 network: float dense, then binary dense layers, BN + sign in between."""

    def __init__(self, layers, batch: int, eps: float, device="cuda", fused: bool = True,
                 first_layer: str = "float", engine: int = esp.ENGINE_XOR_POPCOUNT,
                 keep_first_pre: bool = False, packed_first_weights: bool = False):
        self.batch = batch
        self.keep_first_pre = keep_first_pre   # also write the first layer's float pre-activations
        self.engine = engine    # units that evaluate the fused binary layers (esp_engine)
        # "float": fp32 first layer on real-valued input; "bitplane": 8-bit input split into
        # bit-planes and run through the binary product (Sec. 4.3, Eq. 3), exact in integers
        self.first_layer = first_layer
        self.fused = fused      # False: keep every int32 pre-activation (for layer-wise checks)
        self.sizes = [layers[0]["w"].shape[1]] + [l["w"].shape[0] for l in layers]
        bitplane = first_layer == "bitplane"
        # the float first layer's +-1 weights as floats (12.25 MiB for 4096 x 784) or bit-packed
        # like every other layer's (0.4 MiB; Sec. 6.2 "Binary optimized layers"): same speed
        self.packed_first_weights = packed_first_weights and not bitplane
        if self.packed_first_weights:
            self.w1, self.w1_bits = None, _pack_weights(layers[0]["w"], device)
        else:
            self.w1, self.w1_bits = _dev_f32(layers[0]["w"], device), None
        # the bit-plane layer as one matrix-core call (planes combined in the product's epilogue)
        # when the engine allows the matrix cores and the batch gives them enough tiles
        self.bitplane_fused = bitplane and fused and (
            engine == esp.ENGINE_MFMA or (engine == esp.ENGINE_AUTO and batch >= 64))
        self.bn = [_FoldedBN(l["bn"], eps, device, integer=(i > 0 or bitplane)) if l["bn"] is not None else None
                   for i, l in enumerate(layers)]
        self.wp = [None] + [_pack_weights(l["w"], device) for l in layers[1:]]
        if bitplane:
            self.wp[0] = _pack_weights(layers[0]["w"], device)
            self.wsum0 = esp.row_sums(self.wp[0], self.sizes[0])
            self.planes = torch.empty((batch, 8, esp.words(self.sizes[0])), dtype=esp.PACKED, device=device)
            self.plane_dots = torch.empty((batch, 8, self.sizes[1]), dtype=torch.int32, device=device)
        # pre-allocated activations
        self.pre = [torch.empty((batch, self.sizes[1]), dtype=torch.int32 if bitplane else torch.float32,
                                device=device)]
        self.pre += [torch.empty((batch, n), dtype=torch.int32, device=device) for n in self.sizes[2:]]
        self.act = [torch.empty((batch, esp.words(n)), dtype=esp.PACKED, device=device)
                    for n in self.sizes[1:-1]]
        torch.cuda.synchronize()

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        if self.first_layer == "bitplane" and self.bitplane_fused:
            # planes, then ONE call: product of the planes, their combination and the threshold
            esp.bitplane_pack_u8(x, out=self.planes)
            esp.bitplane_dense(self.planes, self.wp[0], self.wsum0, self.sizes[0], thr=self.bn[0].thr,
                               flip=self.bn[0].flip, bits=self.act[0],
                               y=self.pre[0] if self.keep_first_pre else None)
        elif self.first_layer == "bitplane":
            esp.bitplane_pack_u8(x, out=self.planes)
            esp.bgemm(self.planes.view(self.batch * 8, -1), self.wp[0], self.sizes[0],
                      out=self.plane_dots.view(self.batch * 8, -1))
            esp.bitplane_combine(self.plane_dots, self.wsum0, out=self.pre[0])
            esp.bn_sign_pack(self.pre[0], self.bn[0].thr, self.bn[0].flip, out=self.act[0])
        elif self.packed_first_weights:
            esp.dense_f32_bw_bn_sign_pack(x, self.w1_bits, self.bn[0].thr, self.bn[0].sgn, out=self.act[0],
                                          pre=self.pre[0] if self.keep_first_pre else None)
        else:
            # one kernel; the float pre-activations are written only when asked for
            esp.dense_f32_bn_sign_pack(x, self.w1, self.bn[0].thr, self.bn[0].sgn, out=self.act[0],
                                       pre=self.pre[0] if self.keep_first_pre else None)
        self._binary_layers()
        return self.pre[-1]

    def _binary_layers(self):
        for i in range(1, len(self.wp)):
            if self.bn[i] is None:
                esp.bgemm(self.act[i - 1], self.wp[i], self.sizes[i], out=self.pre[i])
            elif self.fused:
                # threshold + sign + pack in the product's epilogue: no int32 round trip
                esp.bgemm_bn_sign_pack(self.act[i - 1], self.wp[i], self.sizes[i], self.bn[i].thr,
                                       self.bn[i].flip, out=self.act[i], engine=self.engine)
            else:
                esp.bgemm(self.act[i - 1], self.wp[i], self.sizes[i], out=self.pre[i])
                esp.bn_sign_pack(self.pre[i], self.bn[i].thr, self.bn[i].flip, out=self.act[i])

    def forward_from_first_act(self, act0: torch.Tensor) -> torch.Tensor:
        """Binary layers only, starting from given packed first-layer activations."""
        self.act[0].copy_(act0)
        self._binary_layers()
        return self.pre[-1]


class BinaryCNN:
    """Sec. 6.3 network: float conv, binary 3x3 convs (border = -1), OR max-pools, binary dense."""

    def __init__(self, layers, batch: int, eps: float, hw: int = 32, device="cuda",
                 keep_first_pre: bool = False, fused: bool = True, zero_pad: bool = False,
                 engine: int = esp.ENGINE_XOR_POPCOUNT, fuse_pool: bool = True):
        self.batch = batch
        self.engine = engine    # units that evaluate the fused binary layers (esp_engine)
        # zero_pad: add the load-time correction matrix (Sec. 5.2 "Zero-padding for
        # convolutions") after every binary convolution, i.e. true zero padding
        self.zero_pad = zero_pad
        if zero_pad:
            fused = False
        self.keep_first_pre = keep_first_pre   # also write the first layer's float pre-activations
        self.fused = fused      # False: keep every int32 pre-activation (for layer-wise checks)
        self.fuse_pool = fuse_pool and fused   # OR max-pool inside the preceding convolution's epilogue
        self.steps = []          # one record per layer, in order
        h = hw
        c = layers[0]["w"].shape[3]
        flat = None
        ws_bytes = 16
        for i, l in enumerate(layers):
            kind = l["kind"]
            rec = {"kind": kind}
            if kind == "pool":
                rec.update(c=c, h=h)
                prev = self.steps[-1]
                # a binary convolution right before the pool takes it into its own epilogue
                rec["fused_into_conv"] = bool(self.fuse_pool and i > 1 and prev["kind"] == "conv" and
                                              esp.bconv_pool2_fusable(h, h, prev["c"], 3, 3, 1, 1))
                prev["pool_after"] = rec["fused_into_conv"]
                h //= 2
                rec["out"] = torch.empty((batch, h, h, esp.words(c)), dtype=esp.PACKED, device=device)
            elif kind == "conv":
                l2 = l["w"].shape[0]
                rec.update(c=c, h=h, l2=l2)
                if i == 0:
                    rec["w"] = _dev_f32(l["w"], device)
                    rec["pre"] = torch.empty((batch, h, h, l2), dtype=torch.float32, device=device)
                    rec["bn"] = _FoldedBN(l["bn"], eps, device, integer=False)
                else:
                    rec["w"] = _pack_weights(l["w"], device)
                    rec["pre"] = torch.empty((batch, h, h, l2), dtype=torch.int32, device=device)
                    rec["bn"] = _FoldedBN(l["bn"], eps, device)
                    ws_bytes = max(ws_bytes, esp.bconv_workspace_bytes(batch, h, h, c, 3, 3, 1, 1))
                    if zero_pad:
                        rec["corr"] = esp.pad_correction(rec["w"], c, h, h, 1, 1)
                rec["out"] = torch.empty((batch, h, h, esp.words(l2)), dtype=esp.PACKED, device=device)
                c = l2
            else:
                n, k = l["w"].shape
                if flat is None:
                    flat = h * h * c
                    assert flat == k, (flat, k)
                rec.update(k=k, n=n)
                rec["w"] = _pack_weights(l["w"], device)
                rec["pre"] = torch.empty((batch, n), dtype=torch.int32, device=device)
                if l["bn"] is not None:
                    rec["bn"] = _FoldedBN(l["bn"], eps, device)
                    rec["out"] = torch.empty((batch, esp.words(n)), dtype=esp.PACKED, device=device)
                else:
                    rec["bn"] = None
            self.steps.append(rec)
        self.workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=device)
        torch.cuda.synchronize()

    def forward(self, x: torch.Tensor, first_act: torch.Tensor | None = None) -> torch.Tensor:
        cur = None
        for i, s in enumerate(self.steps):
            kind = s["kind"]
            if kind == "pool":
                if not s["fused_into_conv"]:
                    cur = esp.bmaxpool(cur, s["c"], 2, 2, out=s["out"])
            elif kind == "conv" and i == 0:
                if first_act is None:
                    esp.conv_f32_bn_sign_pack(x, s["w"], s["bn"].thr, s["bn"].sgn, 1, 1, out=s["out"],
                                              pre=s["pre"] if self.keep_first_pre else None)
                else:
                    s["out"].copy_(first_act)
                cur = s["out"]
            elif kind == "conv":
                if self.fused and s.get("pool_after"):
                    cur = esp.bconv_bn_sign_pack_pool2(cur, s["w"], s["c"], s["bn"].thr, s["bn"].flip, 1, 1,
                                                       out=self.steps[i + 1]["out"], engine=self.engine)
                elif self.fused:
                    cur = esp.bconv_bn_sign_pack(cur, s["w"], s["c"], s["bn"].thr, s["bn"].flip, 1, 1,
                                                 workspace=self.workspace, out=s["out"], engine=self.engine)
                else:
                    esp.bconv(cur, s["w"], s["c"], 1, 1, workspace=self.workspace, out=s["pre"])
                    if self.zero_pad:
                        esp.add_pad_correction(s["pre"], s["corr"], s["h"], s["h"], 3, 3, 1, 1)
                    cur = esp.bn_sign_pack(s["pre"], s["bn"].thr, s["bn"].flip, out=s["out"])
            else:
                a = cur.reshape(self.batch, -1)   # flatten in storage order: free
                if s["bn"] is None:
                    cur = esp.bgemm(a, s["w"], s["k"], out=s["pre"])
                elif self.fused:
                    cur = esp.bgemm_bn_sign_pack(a, s["w"], s["k"], s["bn"].thr, s["bn"].flip, out=s["out"],
                                                 engine=self.engine)
                else:
                    esp.bgemm(a, s["w"], s["k"], out=s["pre"])
                    cur = esp.bn_sign_pack(s["pre"], s["bn"].thr, s["bn"].flip, out=s["out"])
        return cur
