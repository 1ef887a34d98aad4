"""Thin Python binding of the C ABI declared in ``include/espresso_hip.h``.

Argument marshalling only: every function checks dtype / device / contiguity of
its torch tensors, allocates the output tensor when none is passed, and calls
the entry point of the same name on torch's current HIP stream.  All arithmetic
of the method runs in the library's kernels; there is no CPU fallback -- if the
shared library is missing, importing it raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libespresso_hip.so")

ESP_OK = 0
ENGINE_XOR_POPCOUNT = 0
ENGINE_MFMA = 1
ENGINE_AUTO = 2

EXPORTS = (
    "esp_strerror", "esp_version", "esp_pack_f32", "esp_bgemm", "esp_unroll",
    "esp_bconv_workspace_bytes", "esp_bconv", "esp_bn_fold", "esp_bn_sign_pack",
    "esp_bmaxpool", "esp_dense_f32", "esp_conv_f32", "esp_bn_fold_f32", "esp_bn_sign_pack_f32",
    "esp_conv_f32_bn_sign_pack", "esp_bconv_needs_workspace", "esp_bgemm_bn_sign_pack",
    "esp_bconv_bn_sign_pack", "esp_pad_correction", "esp_add_pad_correction",
    "esp_bitplane_pack_u8", "esp_row_sums", "esp_bitplane_combine", "esp_bgemm_mfma", "esp_bconv_mfma",
    "esp_bconv_pool2_fusable", "esp_bconv_bn_sign_pack_pool2", "esp_dense_f32_bn_sign_pack",
    "esp_xor_popcount_probe", "esp_bitplane_dense", "esp_dense_f32_bw_bn_sign_pack", "esp_bconv_noalloc",
)

_lib = None


class EspressoError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


def lib() -> ctypes.CDLL:
    """Load ``libespresso_hip.so`` (built by ``paper_1705_07175_amd.build``); raise if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_1705_07175_amd.build`" % LIB_PATH)
        l = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, f32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
        l.esp_strerror.restype = ctypes.c_char_p
        l.esp_strerror.argtypes = [i32]
        l.esp_version.restype = i32
        l.esp_pack_f32.argtypes = [vp, vp, i64, i64, vp]
        l.esp_bgemm.argtypes = [vp, vp, vp, i64, i64, i64, vp]
        l.esp_unroll.argtypes = [vp, vp] + [i32] * 8 + [vp]
        l.esp_bconv_workspace_bytes.restype = ctypes.c_size_t
        l.esp_bconv_workspace_bytes.argtypes = [i32] * 8
        l.esp_bconv.argtypes = [vp, vp, vp] + [i32] * 9 + [vp, ctypes.c_size_t, vp]
        l.esp_bconv_noalloc.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
        l.esp_bn_fold.argtypes = [vp, vp, vp, vp, f32, i32, vp, vp]
        l.esp_bn_sign_pack.argtypes = [vp, vp, vp, vp, i64, i32, vp]
        l.esp_bmaxpool.argtypes = [vp, vp] + [i32] * 6 + [vp]
        l.esp_dense_f32.argtypes = [vp, vp, vp, i64, i64, i64, vp]
        l.esp_conv_f32.argtypes = [vp, vp, vp] + [i32] * 9 + [vp]
        l.esp_bn_fold_f32.argtypes = [vp, vp, vp, vp, f32, i32, vp, vp]
        l.esp_bn_sign_pack_f32.argtypes = [vp, vp, vp, vp, i64, i32, vp]
        l.esp_conv_f32_bn_sign_pack.argtypes = [vp, vp, vp, vp, vp, vp] + [i32] * 9 + [vp]
        l.esp_bconv_needs_workspace.argtypes = [i32]
        l.esp_bgemm_bn_sign_pack.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp]
        l.esp_bconv_bn_sign_pack.argtypes = [vp, vp, vp, vp, vp] + [i32] * 9 + [vp, ctypes.c_size_t, i32, vp]
        l.esp_bconv_mfma.argtypes = [vp, vp, vp] + [i32] * 9 + [vp, ctypes.c_size_t, vp]
        l.esp_pad_correction.argtypes = [vp, vp] + [i32] * 8 + [vp]
        l.esp_add_pad_correction.argtypes = [vp, vp] + [i32] * 8 + [vp]
        l.esp_bitplane_pack_u8.argtypes = [vp, vp, i64, i64, i64, vp]
        l.esp_row_sums.argtypes = [vp, vp, i64, i64, i64, vp]
        l.esp_bitplane_combine.argtypes = [vp, vp, vp, i64, i64, i64, vp]
        l.esp_bgemm_mfma.argtypes = [vp, vp, vp, i64, i64, i64, vp]
        l.esp_bconv_pool2_fusable.argtypes = [i32] * 7
        l.esp_bconv_bn_sign_pack_pool2.argtypes = [vp, vp, vp, vp, vp] + [i32] * 9 + [i32, vp]
        l.esp_dense_f32_bn_sign_pack.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp]
        l.esp_dense_f32_bw_bn_sign_pack.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp]
        l.esp_xor_popcount_probe.argtypes = [vp, i32, i32, i32, vp, vp]
        l.esp_bitplane_dense.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, vp]
        l.esp_version.argtypes = []
        for name in EXPORTS:
            # without a prototype ctypes would pass pointers as 32-bit ints: refuse to load
            if getattr(l, name).argtypes is None:
                raise ImportError("binding.py declares no argument types for %s" % name)
            if name not in ("esp_strerror", "esp_bconv_workspace_bytes"):
                getattr(l, name).restype = i32
        _lib = l
    return _lib


def strerror(status: int) -> str:
    return lib().esp_strerror(int(status)).decode()


def version() -> int:
    return int(lib().esp_version())


def _check(status: int, where: str) -> None:
    if status != ESP_OK:
        raise EspressoError(status, where)


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t: torch.Tensor, dtype: torch.dtype, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a device tensor" % name)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t.data_ptr()


def _out(out, shape, dtype: torch.dtype, device) -> torch.Tensor:
    """The result buffer: a fresh one, or the caller's after a size check (the kernels trust it)."""
    shape = tuple(int(d) for d in shape)
    if out is None:
        return torch.empty(shape, dtype=dtype, device=device)
    n = 1
    for d in shape:
        n *= d
    if out.numel() != n:
        raise ValueError("out has %d elements, the result has %d %s" % (out.numel(), n, shape))
    return out


def words(k: int) -> int:
    """64-bit words per packed row of ``k`` values."""
    return (int(k) + 63) // 64


# torch has no uint64 arithmetic, and none is needed: packed buffers are int64 tensors
# that are only ever handed to the library (same bytes as uint64).
PACKED = torch.int64


def pack_f32(src: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_pack_f32``: float [..., k] -> packed words [..., ceil(k/64)] (sign, Eq. 1)."""
    p = _dev(src, torch.float32, "src")
    k = src.shape[-1]
    rows = src.numel() // k if k else 0
    out = _out(out, src.shape[:-1] + (words(k),), PACKED, src.device)
    _check(lib().esp_pack_f32(p, _dev(out, PACKED, "out"), rows, k, _stream()), "esp_pack_f32")
    return out


def bgemm(a: torch.Tensor, b: torch.Tensor, k: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_bgemm``: packed A [M][Kw], packed B [N][Kw], true length k -> int32 [M][N] (Eq. 2)."""
    pa, pb = _dev(a, PACKED, "a"), _dev(b, PACKED, "b")
    M, N = a.shape[0], b.shape[0]
    if a.dim() != 2 or b.dim() != 2 or a.shape[1] != words(k) or b.shape[1] != words(k):
        raise ValueError("a and b must be [rows][ceil(k/64)]")
    out = _out(out, (M, N), torch.int32, a.device)
    _check(lib().esp_bgemm(pa, pb, _dev(out, torch.int32, "out"), M, N, int(k), _stream()), "esp_bgemm")
    return out


def bgemm_mfma(a: torch.Tensor, b: torch.Tensor, k: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_bgemm_mfma``: same result as :func:`bgemm`, computed on the matrix cores."""
    pa, pb = _dev(a, PACKED, "a"), _dev(b, PACKED, "b")
    M, N = a.shape[0], b.shape[0]
    if a.dim() != 2 or b.dim() != 2 or a.shape[1] != words(k) or b.shape[1] != words(k):
        raise ValueError("a and b must be [rows][ceil(k/64)]")
    out = _out(out, (M, N), torch.int32, a.device)
    _check(lib().esp_bgemm_mfma(pa, pb, _dev(out, torch.int32, "out"), M, N, int(k), _stream()),
           "esp_bgemm_mfma")
    return out


def conv_out(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


def unroll(x: torch.Tensor, c: int, kh: int, kw: int, stride: int, pad: int,
           out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_unroll``: packed NHWC [B][H][W][Cw] -> lowered matrix [B*H2*W2][kh*kw*Cw] (Fig. 3)."""
    p = _dev(x, PACKED, "x")
    B, H, W, Cw = x.shape
    if Cw != words(c):
        raise ValueError("last dim must be ceil(c/64)")
    H2, W2 = conv_out(H, kh, stride, pad), conv_out(W, kw, stride, pad)
    out = _out(out, (B * max(H2, 0) * max(W2, 0), kh * kw * Cw), PACKED, x.device)
    _check(lib().esp_unroll(p, _dev(out, PACKED, "out"), B, H, W, int(c), kh, kw, stride, pad, _stream()),
           "esp_unroll")
    return out


def bconv_workspace_bytes(B, H, W, c, kh, kw, stride, pad) -> int:
    return int(lib().esp_bconv_workspace_bytes(B, H, W, int(c), kh, kw, stride, pad))


def bconv(x: torch.Tensor, filt: torch.Tensor, c: int, stride: int, pad: int,
          workspace: torch.Tensor | None = None, out: torch.Tensor | None = None,
          engine: int = ENGINE_XOR_POPCOUNT) -> torch.Tensor:
    """``esp_bconv``: packed NHWC x, packed filters [L2][kh][kw][Cw] -> int32 [B][H2][W2][L2]."""
    px, pf = _dev(x, PACKED, "x"), _dev(filt, PACKED, "filt")
    B, H, W, Cw = x.shape
    L2, kh, kw, Cw2 = filt.shape
    if Cw != words(c) or Cw2 != Cw:
        raise ValueError("channel words mismatch")
    H2, W2 = conv_out(H, kh, stride, pad), conv_out(W, kw, stride, pad)
    if workspace is None:
        need = bconv_workspace_bytes(B, H, W, c, kh, kw, stride, pad)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    out = _out(out, (B, max(H2, 0), max(W2, 0), L2), torch.int32, x.device)
    fn = lib().esp_bconv_mfma if engine == ENGINE_MFMA else lib().esp_bconv
    _check(fn(px, pf, _dev(out, torch.int32, "out"), B, H, W, int(c), L2, kh, kw, stride, pad,
              _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream()),
           "esp_bconv_mfma" if engine == ENGINE_MFMA else "esp_bconv")
    return out


BCONV_NOALLOC_MAX_BYTES = 16 << 20


def bconv_noalloc(x: torch.Tensor, filt: torch.Tensor, c: int, stride: int, pad: int,
                  out: torch.Tensor) -> torch.Tensor:
    """``esp_bconv_noalloc``: :func:`bconv` without a workspace (the lowered matrix goes to the
    library's fixed scratch array).  ``out`` is required: nothing is allocated on this path."""
    px, pf = _dev(x, PACKED, "x"), _dev(filt, PACKED, "filt")
    B, H, W, Cw = x.shape
    L2, kh, kw, Cw2 = filt.shape
    if Cw != words(c) or Cw2 != Cw:
        raise ValueError("channel words mismatch")
    H2, W2 = conv_out(H, kh, stride, pad), conv_out(W, kw, stride, pad)
    if out is None or out.numel() != B * max(H2, 0) * max(W2, 0) * L2:
        raise ValueError("out must be the caller's int32 [B][H2][W2][L2] buffer")
    _check(lib().esp_bconv_noalloc(px, pf, _dev(out, torch.int32, "out"), B, H, W, int(c), L2, kh, kw, stride, pad,
                                   _stream()), "esp_bconv_noalloc")
    return out


def bconv_needs_workspace(c: int) -> bool:
    return bool(lib().esp_bconv_needs_workspace(int(c)))


def bgemm_bn_sign_pack(a: torch.Tensor, b: torch.Tensor, k: int, thr: torch.Tensor, flip: torch.Tensor,
                       out: torch.Tensor | None = None, engine: int = ENGINE_XOR_POPCOUNT) -> torch.Tensor:
    """``esp_bgemm_bn_sign_pack``: product + folded threshold + sign -> packed [M][ceil(N/64)]."""
    pa, pb = _dev(a, PACKED, "a"), _dev(b, PACKED, "b")
    M, N = a.shape[0], b.shape[0]
    if a.dim() != 2 or b.dim() != 2 or a.shape[1] != words(k) or b.shape[1] != words(k):
        raise ValueError("a and b must be [rows][ceil(k/64)]")
    if thr.numel() != N or flip.numel() != words(N):
        raise ValueError("thr/flip size mismatch")
    out = _out(out, (M, words(N)), PACKED, a.device)
    _check(lib().esp_bgemm_bn_sign_pack(pa, pb, _dev(thr, torch.int32, "thr"), _dev(flip, PACKED, "flip"),
                                        _dev(out, PACKED, "out"), M, N, int(k), int(engine), _stream()),
           "esp_bgemm_bn_sign_pack")
    return out


def bconv_bn_sign_pack(x: torch.Tensor, filt: torch.Tensor, c: int, thr: torch.Tensor, flip: torch.Tensor,
                       stride: int, pad: int, workspace: torch.Tensor | None = None,
                       out: torch.Tensor | None = None, engine: int = ENGINE_XOR_POPCOUNT) -> torch.Tensor:
    """``esp_bconv_bn_sign_pack``: convolution + folded threshold + sign -> packed NHWC bits."""
    px, pf = _dev(x, PACKED, "x"), _dev(filt, PACKED, "filt")
    B, H, W, Cw = x.shape
    L2, kh, kw, Cw2 = filt.shape
    if Cw != words(c) or Cw2 != Cw or thr.numel() != L2 or flip.numel() != words(L2):
        raise ValueError("shape mismatch")
    H2, W2 = conv_out(H, kh, stride, pad), conv_out(W, kw, stride, pad)
    if workspace is None and bconv_needs_workspace(c):
        need = bconv_workspace_bytes(B, H, W, c, kh, kw, stride, pad)
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=x.device)
    out = _out(out, (B, max(H2, 0), max(W2, 0), words(L2)), PACKED, x.device)
    ws_ptr = _dev(workspace, torch.uint8, "workspace") if workspace is not None else None
    ws_len = workspace.numel() if workspace is not None else 0
    _check(lib().esp_bconv_bn_sign_pack(px, pf, _dev(thr, torch.int32, "thr"), _dev(flip, PACKED, "flip"),
                                        _dev(out, PACKED, "out"), B, H, W, int(c), L2, kh, kw, stride, pad,
                                        ws_ptr, ws_len, int(engine), _stream()), "esp_bconv_bn_sign_pack")
    return out


def bconv_pool2_fusable(h: int, w: int, c: int, kh: int, kw: int, stride: int, pad: int) -> bool:
    """``esp_bconv_pool2_fusable``: can the 2x2 max-pool be fused behind this convolution?"""
    return bool(lib().esp_bconv_pool2_fusable(int(h), int(w), int(c), int(kh), int(kw), int(stride), int(pad)))


def bconv_bn_sign_pack_pool2(x: torch.Tensor, filt: torch.Tensor, c: int, thr: torch.Tensor,
                             flip: torch.Tensor, stride: int, pad: int, out: torch.Tensor | None = None,
                             engine: int = ENGINE_XOR_POPCOUNT) -> torch.Tensor:
    """``esp_bconv_bn_sign_pack_pool2``: convolution + threshold + sign + 2x2 OR max-pool."""
    px, pf = _dev(x, PACKED, "x"), _dev(filt, PACKED, "filt")
    B, H, W, Cw = x.shape
    L2, kh, kw, Cw2 = filt.shape
    if Cw != words(c) or Cw2 != Cw or thr.numel() != L2 or flip.numel() != words(L2):
        raise ValueError("shape mismatch")
    H2, W2 = conv_out(H, kh, stride, pad), conv_out(W, kw, stride, pad)
    out = _out(out, (B, max(H2, 0) // 2, max(W2, 0) // 2, words(L2)), PACKED, x.device)
    _check(lib().esp_bconv_bn_sign_pack_pool2(px, pf, _dev(thr, torch.int32, "thr"), _dev(flip, PACKED, "flip"),
                                              _dev(out, PACKED, "out"), B, H, W, int(c), L2, kh, kw, stride,
                                              pad, int(engine), _stream()), "esp_bconv_bn_sign_pack_pool2")
    return out


def pad_correction(filt: torch.Tensor, c: int, h: int, w: int, stride: int, pad: int,
                   out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_pad_correction``: packed filters [L2][kh][kw][Cw] -> int32 correction [H2][W2][L2]."""
    pf = _dev(filt, PACKED, "filt")
    L2, kh, kw, Cw = filt.shape
    if Cw != words(c):
        raise ValueError("channel words mismatch")
    H2, W2 = conv_out(h, kh, stride, pad), conv_out(w, kw, stride, pad)
    out = _out(out, (max(H2, 0), max(W2, 0), L2), torch.int32, filt.device)
    _check(lib().esp_pad_correction(pf, _dev(out, torch.int32, "out"), h, w, int(c), L2, kh, kw, stride, pad,
                                    _stream()), "esp_pad_correction")
    return out


def add_pad_correction(x: torch.Tensor, corr: torch.Tensor, h: int, w: int, kh: int, kw: int,
                       stride: int, pad: int) -> torch.Tensor:
    """``esp_add_pad_correction``: x int32 [B][H2][W2][L2] += corr [H2][W2][L2], in place."""
    B, H2, W2, L2 = x.shape
    if tuple(corr.shape) != (H2, W2, L2) or (H2, W2) != (conv_out(h, kh, stride, pad), conv_out(w, kw, stride, pad)):
        raise ValueError("correction shape mismatch")
    _check(lib().esp_add_pad_correction(_dev(x, torch.int32, "x"), _dev(corr, torch.int32, "corr"), B, h, w,
                                        L2, kh, kw, stride, pad, _stream()), "esp_add_pad_correction")
    return x


def bn_fold(gamma, beta, mean, var, eps: float):
    """``esp_bn_fold`` (host): float32 numpy parameters -> (thr int32 [C], flip uint64 [Cw])."""
    g, b, m, v = (np.ascontiguousarray(t, dtype=np.float32) for t in (gamma, beta, mean, var))
    C = g.shape[0]
    thr = np.empty(C, dtype=np.int32)
    flip = np.empty(words(C), dtype=np.uint64)
    _check(lib().esp_bn_fold(g.ctypes.data, b.ctypes.data, m.ctypes.data, v.ctypes.data,
                             ctypes.c_float(eps), C, thr.ctypes.data, flip.ctypes.data), "esp_bn_fold")
    return thr, flip


def bn_sign_pack(x: torch.Tensor, thr: torch.Tensor, flip: torch.Tensor,
                 out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_bn_sign_pack``: int32 [..., C] + folded thresholds -> packed [..., Cw]."""
    px = _dev(x, torch.int32, "x")
    C = x.shape[-1]
    rows = x.numel() // C if C else 0
    if thr.numel() != C or flip.numel() != words(C):
        raise ValueError("thr/flip size mismatch")
    out = _out(out, x.shape[:-1] + (words(C),), PACKED, x.device)
    _check(lib().esp_bn_sign_pack(px, _dev(thr, torch.int32, "thr"), _dev(flip, PACKED, "flip"),
                                  _dev(out, PACKED, "out"), rows, C, _stream()), "esp_bn_sign_pack")
    return out


def bmaxpool(x: torch.Tensor, c: int, win: int = 2, stride: int = 2,
             out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_bmaxpool``: packed NHWC -> packed NHWC, max of +-1 values as bitwise OR."""
    p = _dev(x, PACKED, "x")
    B, H, W, Cw = x.shape
    if Cw != words(c):
        raise ValueError("last dim must be ceil(c/64)")
    H2, W2 = (H - win) // stride + 1, (W - win) // stride + 1
    out = _out(out, (B, max(H2, 0), max(W2, 0), Cw), PACKED, x.device)
    _check(lib().esp_bmaxpool(p, _dev(out, PACKED, "out"), B, H, W, int(c), win, stride, _stream()),
           "esp_bmaxpool")
    return out


def dense_f32(x: torch.Tensor, w: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_dense_f32``: float [M][K] times float +-1 weights [N][K] -> float [M][N]."""
    px, pw = _dev(x, torch.float32, "x"), _dev(w, torch.float32, "w")
    M, K = x.shape
    N, K2 = w.shape
    if K != K2:
        raise ValueError("K mismatch")
    out = _out(out, (M, N), torch.float32, x.device)
    _check(lib().esp_dense_f32(px, pw, _dev(out, torch.float32, "out"), M, N, K, _stream()), "esp_dense_f32")
    return out


def dense_f32_bn_sign_pack(x: torch.Tensor, w: torch.Tensor, thr: torch.Tensor, sgn: torch.Tensor,
                           out: torch.Tensor | None = None, pre: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_dense_f32_bn_sign_pack``: float dense layer + folded batch-norm + sign -> packed [M][Nw].
    ``pre`` (float [M][N]) receives the pre-activations if given."""
    px, pw = _dev(x, torch.float32, "x"), _dev(w, torch.float32, "w")
    M, K = x.shape
    N, K2 = w.shape
    if K != K2 or thr.numel() != N or sgn.numel() != N:
        raise ValueError("shape mismatch")
    out = _out(out, (M, words(N)), PACKED, x.device)
    if pre is not None:
        _out(pre, (M, N), torch.float32, x.device)
    ppre = _dev(pre, torch.float32, "pre") if pre is not None else None
    _check(lib().esp_dense_f32_bn_sign_pack(px, pw, _dev(thr, torch.float32, "thr"), _dev(sgn, torch.float32, "sgn"),
                                            _dev(out, PACKED, "out"), ppre, M, N, K, _stream()),
           "esp_dense_f32_bn_sign_pack")
    return out


def dense_f32_bw_bn_sign_pack(x: torch.Tensor, wbits: torch.Tensor, thr: torch.Tensor, sgn: torch.Tensor,
                              out: torch.Tensor | None = None, pre: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_dense_f32_bw_bn_sign_pack``: the float dense layer with bit-packed +-1 weights
    (``wbits`` packed [N][ceil(K/64)] as from ``pack_f32``) + folded batch-norm + sign."""
    px, pw = _dev(x, torch.float32, "x"), _dev(wbits, PACKED, "wbits")
    M, K = x.shape
    N = wbits.shape[0]
    if wbits.dim() != 2 or wbits.shape[1] != words(K) or thr.numel() != N or sgn.numel() != N:
        raise ValueError("shape mismatch")
    out = _out(out, (M, words(N)), PACKED, x.device)
    if pre is not None:
        _out(pre, (M, N), torch.float32, x.device)
    ppre = _dev(pre, torch.float32, "pre") if pre is not None else None
    _check(lib().esp_dense_f32_bw_bn_sign_pack(px, pw, _dev(thr, torch.float32, "thr"),
                                               _dev(sgn, torch.float32, "sgn"), _dev(out, PACKED, "out"), ppre,
                                               M, N, K, _stream()),
           "esp_dense_f32_bw_bn_sign_pack")
    return out


def conv_f32(x: torch.Tensor, filt: torch.Tensor, stride: int, pad: int,
             out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_conv_f32``: float NHWC, float +-1 filters [L2][kh][kw][C], zero padding."""
    px, pf = _dev(x, torch.float32, "x"), _dev(filt, torch.float32, "filt")
    B, H, W, C = x.shape
    L2, kh, kw, C2 = filt.shape
    if C != C2:
        raise ValueError("C mismatch")
    H2, W2 = conv_out(H, kh, stride, pad), conv_out(W, kw, stride, pad)
    out = _out(out, (B, max(H2, 0), max(W2, 0), L2), torch.float32, x.device)
    _check(lib().esp_conv_f32(px, pf, _dev(out, torch.float32, "out"), B, H, W, C, L2, kh, kw, stride, pad,
                              _stream()), "esp_conv_f32")
    return out


def bn_fold_f32(gamma, beta, mean, var, eps: float):
    """``esp_bn_fold_f32`` (host): float32 numpy parameters -> (thr float32 [C], sgn float32 [C])."""
    g, b, m, v = (np.ascontiguousarray(t, dtype=np.float32) for t in (gamma, beta, mean, var))
    C = g.shape[0]
    thr = np.empty(C, dtype=np.float32)
    sgn = np.empty(C, dtype=np.float32)
    _check(lib().esp_bn_fold_f32(g.ctypes.data, b.ctypes.data, m.ctypes.data, v.ctypes.data,
                                 ctypes.c_float(eps), C, thr.ctypes.data, sgn.ctypes.data), "esp_bn_fold_f32")
    return thr, sgn


def bn_sign_pack_f32(x: torch.Tensor, thr: torch.Tensor, sgn: torch.Tensor,
                     out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_bn_sign_pack_f32``: float [..., C] + folded float thresholds -> packed [..., Cw]."""
    px = _dev(x, torch.float32, "x")
    C = x.shape[-1]
    rows = x.numel() // C if C else 0
    if thr.numel() != C or sgn.numel() != C:
        raise ValueError("thr/sgn size mismatch")
    out = _out(out, x.shape[:-1] + (words(C),), PACKED, x.device)
    _check(lib().esp_bn_sign_pack_f32(px, _dev(thr, torch.float32, "thr"), _dev(sgn, torch.float32, "sgn"),
                                      _dev(out, PACKED, "out"), rows, C, _stream()), "esp_bn_sign_pack_f32")
    return out


def conv_f32_bn_sign_pack(x: torch.Tensor, filt: torch.Tensor, thr: torch.Tensor, sgn: torch.Tensor,
                          stride: int, pad: int, out: torch.Tensor | None = None,
                          pre: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_conv_f32_bn_sign_pack``: float conv + folded batch-norm + sign + pack in one pass.
    ``pre`` (float [B][H2][W2][L2]) receives the pre-activations if given."""
    px, pf = _dev(x, torch.float32, "x"), _dev(filt, torch.float32, "filt")
    B, H, W, C = x.shape
    L2, kh, kw, C2 = filt.shape
    if C != C2 or thr.numel() != L2 or sgn.numel() != L2:
        raise ValueError("shape mismatch")
    H2, W2 = conv_out(H, kh, stride, pad), conv_out(W, kw, stride, pad)
    out = _out(out, (B, max(H2, 0), max(W2, 0), words(L2)), PACKED, x.device)
    if pre is not None:
        _out(pre, (B, max(H2, 0), max(W2, 0), L2), torch.float32, x.device)
    ppre = _dev(pre, torch.float32, "pre") if pre is not None else None
    _check(lib().esp_conv_f32_bn_sign_pack(px, pf, _dev(thr, torch.float32, "thr"),
                                           _dev(sgn, torch.float32, "sgn"), _dev(out, PACKED, "out"), ppre,
                                           B, H, W, C, L2, kh, kw, stride, pad, _stream()),
           "esp_conv_f32_bn_sign_pack")
    return out


def bitplane_pack_u8(x: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_bitplane_pack_u8``: uint8 [outer][k] -> [outer][8][Kw], or uint8 NHWC [B][H][W][C] ->
    [B][8][H][W][Cw] (each plane a packed NHWC image)."""
    p = _dev(x, torch.uint8, "x")
    k = x.shape[-1]
    outer = x.shape[0]
    inner = x.numel() // (outer * k) if outer and k else 1
    out = _out(out, (outer, 8) + tuple(x.shape[1:-1]) + (words(k),), PACKED, x.device)
    _check(lib().esp_bitplane_pack_u8(p, _dev(out, PACKED, "out"), outer, inner, k, _stream()),
           "esp_bitplane_pack_u8")
    return out


def row_sums(w: torch.Tensor, k: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_row_sums``: packed weights [N][...] holding ``k`` true values per row -> int32 [N]."""
    pw = _dev(w, PACKED, "w")
    N = w.shape[0]
    out = _out(out, (N,), torch.int32, w.device)
    _check(lib().esp_row_sums(pw, _dev(out, torch.int32, "out"), N, w.numel() // N, int(k), _stream()),
           "esp_row_sums")
    return out


def bitplane_combine(d: torch.Tensor, wsum: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """``esp_bitplane_combine``: int32 [outer][8][...][N] -> int32 [outer][...][N]."""
    pd = _dev(d, torch.int32, "d")
    outer, N = d.shape[0], d.shape[-1]
    if d.shape[1] != 8 or wsum.numel() != N:
        raise ValueError("d must be [outer][8][...][N]")
    inner = d.numel() // (outer * 8 * N) if outer else 1
    out = _out(out, (outer,) + tuple(d.shape[2:]), torch.int32, d.device)
    _check(lib().esp_bitplane_combine(pd, _dev(wsum, torch.int32, "wsum"), _dev(out, torch.int32, "out"),
                                      outer, inner, N, _stream()), "esp_bitplane_combine")
    return out


def bitplane_dense(planes: torch.Tensor, w: torch.Tensor, wsum: torch.Tensor, k: int,
                   thr: torch.Tensor | None = None, flip: torch.Tensor | None = None,
                   bits: torch.Tensor | None = None, y: torch.Tensor | None = None, want_y: bool = False):
    """``esp_bitplane_dense``: planes [rows][8][Kw] x W [N][Kw] -> (bits [rows][Nw] if thr is given, y
    int32 [rows][N] if asked for)."""
    pp, pw = _dev(planes, PACKED, "planes"), _dev(w, PACKED, "w")
    rows, N = planes.shape[0], w.shape[0]
    if planes.shape[1] != 8 or wsum.numel() != N:
        raise ValueError("planes must be [rows][8][Kw], wsum one value per row of w")
    if thr is not None:
        bits = _out(bits, (rows, words(N)), PACKED, planes.device)
    if want_y or y is not None:
        y = _out(y, (rows, N), torch.int32, planes.device)
    _check(lib().esp_bitplane_dense(pp, pw, _dev(wsum, torch.int32, "wsum"),
                                    _dev(thr, torch.int32, "thr") if thr is not None else None,
                                    _dev(flip, PACKED, "flip") if thr is not None else None,
                                    _dev(bits, PACKED, "bits") if thr is not None else None,
                                    _dev(y, torch.int32, "y") if y is not None else None,
                                    rows, N, int(k), _stream()), "esp_bitplane_dense")
    return bits, y


PROBE_PAIR, PROBE_XOR_ONLY, PROBE_POPCOUNT_ONLY = 0, 1, 2


def xor_popcount_probe(sink: torch.Tensor, blocks: int, iters: int, mode: int = PROBE_PAIR) -> int:
    """``esp_xor_popcount_probe``: launch the in-register xor + popcount loop (or one of the two
    instructions alone); returns the work of the launch: binary operations for ``PROBE_PAIR``, lane
    instructions for the other modes.  ``sink``: uint32/int32 [blocks * 256] on the device."""
    if sink.numel() < blocks * 256:
        raise ValueError("sink must hold blocks * 256 values")
    work = ctypes.c_int64(0)
    _check(lib().esp_xor_popcount_probe(_dev(sink, torch.int32, "sink"), int(blocks), int(iters), int(mode),
                                        ctypes.addressof(work), _stream()), "esp_xor_popcount_probe")
    return int(work.value)


# ------------------------------------------------------------------ host <-> device helpers
def to_packed_tensor(words_np: np.ndarray, device="cuda") -> torch.Tensor:
    """uint64 numpy words -> device tensor of the same bytes."""
    return torch.from_numpy(np.ascontiguousarray(words_np, dtype=np.uint64).view(np.int64)).to(device)


def packed_to_numpy(t: torch.Tensor) -> np.ndarray:
    """Packed device tensor -> uint64 numpy words."""
    return t.cpu().numpy().view(np.uint64)
