"""CPU oracle for the Espresso binary-network forward path -- TEST INFRASTRUCTURE.

Thin numpy/ctypes front end of ``espresso_oracle.c`` (plain C definitions on
unpacked +-1 values, int32 sums, double floating point).  Only the tests, the
smoke check and the benchmark's ``cpu_baseline`` leg may import this package;
the GPU library never does, and this package never imports the GPU library.

Every function cites the passage of the paper (arXiv 1705.07175) it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "espresso_oracle.c")
_LIB = os.path.join(_HERE, "libespresso_oracle.so")
# The pin tests check themselves by running against deliberately broken builds of the C
# source (tests/test_oracle_mutations.py); this variable points the loader at such a build.
_LIB_OVERRIDE = os.environ.get("ESPRESSO_ORACLE_LIB")

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, no fused multiply-add, OpenMP)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
             "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if _LIB_OVERRIDE:
            _lib = ctypes.CDLL(_LIB_OVERRIDE)
        else:
            build()
            _lib = ctypes.CDLL(_LIB)
        _lib.orc_mismatches_words.restype = ctypes.c_int64
        _lib.orc_bn_value.restype = ctypes.c_double
        _lib.orc_bn_value.argtypes = [ctypes.c_double] + [ctypes.c_float] * 5
    return _lib


def _p(a: np.ndarray):
    return ctypes.c_void_p(a.ctypes.data)


def _i64(v):
    return ctypes.c_int64(int(v))


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


# ----------------------------------------------------------------------------
def set_threads(n: int) -> None:
    """Host threads for the loops over independent output rows (default 1)."""
    _load().orc_set_threads(ctypes.c_int(int(n)))


def get_threads() -> int:
    return int(_load().orc_get_threads())


def max_threads() -> int:
    return int(_load().orc_max_threads())


# ----------------------------------------------------------------------------
def sign(x: np.ndarray) -> np.ndarray:
    """Eq. 1: +1 where x >= 0, else -1 (int8).  float32 or float64 input."""
    lib = _load()
    out = np.empty(x.shape, dtype=np.int8)
    if x.dtype == np.float32:
        xc = _c(x, np.float32)
        lib.orc_sign_f32(_p(xc), _p(out), _i64(xc.size))
    else:
        xc = _c(x, np.float64)
        lib.orc_sign_f64(_p(xc), _p(out), _i64(xc.size))
    return out


def pack_bits(s: np.ndarray) -> np.ndarray:
    """Sec. 4.1 / 4.2: +-1 (int8, last dim K) -> uint64 words [..., ceil(K/64)].

    Element k sits in word k//64, bit k%64, LSB first; tail bits are 0."""
    lib = _load()
    sc = _c(s, np.int8)
    k = sc.shape[-1]
    rows = sc.size // k if k else 0
    out = np.empty(sc.shape[:-1] + ((k + 63) // 64,), dtype=np.uint64)
    lib.orc_pm1_to_words(_p(sc), _p(out), _i64(rows), _i64(k))
    return out


def unpack_bits(w: np.ndarray, k: int) -> np.ndarray:
    """Inverse of :func:`pack_bits`: uint64 words [..., ceil(k/64)] -> int8 +-1 [..., k]."""
    lib = _load()
    wc = _c(w, np.uint64)
    kw = (k + 63) // 64
    assert wc.shape[-1] == kw, (wc.shape, k)
    rows = wc.size // kw
    out = np.empty(wc.shape[:-1] + (k,), dtype=np.int8)
    lib.orc_words_to_pm1(_p(wc), _p(out), _i64(rows), _i64(k))
    return out


def mismatches(a_words: np.ndarray, b_words: np.ndarray) -> int:
    """Positions where two packed rows differ, counted bit by bit (for Eq. 2's identity)."""
    lib = _load()
    a = _c(a_words, np.uint64).ravel()
    b = _c(b_words, np.uint64).ravel()
    assert a.size == b.size
    return int(lib.orc_mismatches_words(_p(a), _p(b), _i64(a.size)))


# ----------------------------------------------------------------------------
def dense_pm1(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Sec. 4.2 (what Eq. 2 evaluates): C[m][n] = sum_k a[m][k] b[n][k], int32.

    ``a`` is [M][K], ``b`` is [N][K] (one neuron per row), both int8 +-1."""
    lib = _load()
    a = _c(a, np.int8)
    b = _c(b, np.int8)
    M, K = a.shape
    N, K2 = b.shape
    assert K == K2
    c = np.empty((M, N), dtype=np.int32)
    lib.orc_dense_pm1(_p(a), _p(b), _p(c), _i64(M), _i64(N), _i64(K))
    return c


def conv_out_size(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


def conv_pm1(x: np.ndarray, f: np.ndarray, stride: int = 1, pad: int = 0,
             pad_value: int = -1) -> np.ndarray:
    """Sec. 5.2 "Convolutional layers" + "Zero-padding": NHWC cross-correlation.

    ``x`` int8 [B][H][W][C], ``f`` int8 [L2][kh][kw][C]; border positions take
    ``pad_value`` (-1 for the binary layers).  Returns int32 [B][H2][W2][L2]."""
    lib = _load()
    x = _c(x, np.int8)
    f = _c(f, np.int8)
    B, H, W, C = x.shape
    L2, kh, kw, C2 = f.shape
    assert C == C2
    H2 = conv_out_size(H, kh, stride, pad)
    W2 = conv_out_size(W, kw, stride, pad)
    out = np.empty((B, H2, W2, L2), dtype=np.int32)
    lib.orc_conv_pm1(_p(x), _p(f), _p(out), _i64(B), _i64(H), _i64(W), _i64(C), _i64(L2),
                     _i64(kh), _i64(kw), _i64(stride), _i64(pad), ctypes.c_int(int(pad_value)))
    return out


def unroll_pm1(x: np.ndarray, kh: int, kw: int, stride: int = 1, pad: int = 0,
               pad_value: int = -1) -> np.ndarray:
    """Fig. 3 (unrolling): NHWC int8 -> lowered matrix [B*H2*W2][kh*kw*C]."""
    lib = _load()
    x = _c(x, np.int8)
    B, H, W, C = x.shape
    H2 = conv_out_size(H, kh, stride, pad)
    W2 = conv_out_size(W, kw, stride, pad)
    out = np.empty((B * H2 * W2, kh * kw * C), dtype=np.int8)
    lib.orc_unroll_pm1(_p(x), _p(out), _i64(B), _i64(H), _i64(W), _i64(C),
                       _i64(kh), _i64(kw), _i64(stride), _i64(pad), ctypes.c_int(int(pad_value)))
    return out


def bn(x: np.ndarray, gamma, beta, mean, var, eps: float) -> np.ndarray:
    """Sec. 5.2 batch-norm layer, inference form, per last-dim channel, in double:
    y = gamma * (x - mean) / sqrt(var + eps) + beta (evaluated left to right)."""
    lib = _load()
    C = x.shape[-1]
    g, b, m, v = (_c(t, np.float32) for t in (gamma, beta, mean, var))
    assert g.shape == b.shape == m.shape == v.shape == (C,)
    rows = x.size // C
    y = np.empty(x.shape, dtype=np.float64)
    if np.issubdtype(x.dtype, np.integer):
        xc = _c(x, np.int32)
        lib.orc_bn_i32(_p(xc), _p(g), _p(b), _p(m), _p(v), ctypes.c_float(eps), _p(y),
                       _i64(rows), _i64(C))
    else:
        xc = _c(x, np.float64)
        lib.orc_bn_f64(_p(xc), _p(g), _p(b), _p(m), _p(v), ctypes.c_float(eps), _p(y),
                       _i64(rows), _i64(C))
    return y


def bn_value(x: float, gamma: float, beta: float, mean: float, var: float, eps: float) -> float:
    """One batch-norm value (same expression as :func:`bn`)."""
    return float(_load().orc_bn_value(float(x), float(gamma), float(beta), float(mean),
                                      float(var), float(eps)))


def maxpool_pm1(x: np.ndarray, win: int = 2, stride: int = 2) -> np.ndarray:
    """Sec. 5.2 pooling layer: max over win x win windows of +-1 NHWC values."""
    lib = _load()
    x = _c(x, np.int8)
    B, H, W, C = x.shape
    H2 = (H - win) // stride + 1
    W2 = (W - win) // stride + 1
    out = np.empty((B, H2, W2, C), dtype=np.int8)
    lib.orc_maxpool_pm1(_p(x), _p(out), _i64(B), _i64(H), _i64(W), _i64(C), _i64(win), _i64(stride))
    return out


def dense_f64(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Sec. 3 float variant of a dense layer: x float32 [M][K], w int8 +-1 [N][K] -> float64."""
    lib = _load()
    x = _c(x, np.float32)
    w = _c(w, np.int8)
    M, K = x.shape
    N, K2 = w.shape
    assert K == K2
    y = np.empty((M, N), dtype=np.float64)
    lib.orc_dense_f64(_p(x), _p(w), _p(y), _i64(M), _i64(N), _i64(K))
    return y


def conv_f64(x: np.ndarray, f: np.ndarray, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Float first conv layer: x float32 NHWC, f int8 +-1 [L2][kh][kw][C], zero padding -> float64."""
    lib = _load()
    x = _c(x, np.float32)
    f = _c(f, np.int8)
    B, H, W, C = x.shape
    L2, kh, kw, C2 = f.shape
    assert C == C2
    H2 = conv_out_size(H, kh, stride, pad)
    W2 = conv_out_size(W, kw, stride, pad)
    out = np.empty((B, H2, W2, L2), dtype=np.float64)
    lib.orc_conv_f64(_p(x), _p(f), _p(out), _i64(B), _i64(H), _i64(W), _i64(C), _i64(L2),
                     _i64(kh), _i64(kw), _i64(stride), _i64(pad))
    return out


def dense_u8(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Sec. 4.3 (the product Eq. 3 re-assembles from bit-planes): x uint8 [M][K], w int8 +-1
    [N][K] -> exact int32 [M][N]."""
    lib = _load()
    x = _c(x, np.uint8)
    w = _c(w, np.int8)
    M, K = x.shape
    N, K2 = w.shape
    assert K == K2
    y = np.empty((M, N), dtype=np.int32)
    lib.orc_dense_u8(_p(x), _p(w), _p(y), _i64(M), _i64(N), _i64(K))
    return y


def conv_u8(x: np.ndarray, f: np.ndarray, stride: int = 1, pad: int = 0) -> np.ndarray:
    """Fixed-precision first conv layer: x uint8 NHWC, f int8 +-1 [L2][kh][kw][C], zero padding,
    exact int32 [B][H2][W2][L2]."""
    lib = _load()
    x = _c(x, np.uint8)
    f = _c(f, np.int8)
    B, H, W, C = x.shape
    L2, kh, kw, C2 = f.shape
    assert C == C2
    H2 = conv_out_size(H, kh, stride, pad)
    W2 = conv_out_size(W, kw, stride, pad)
    out = np.empty((B, H2, W2, L2), dtype=np.int32)
    lib.orc_conv_u8(_p(x), _p(f), _p(out), _i64(B), _i64(H), _i64(W), _i64(C), _i64(L2),
                    _i64(kh), _i64(kw), _i64(stride), _i64(pad))
    return out


def bn_sign(x: np.ndarray, bnp, eps: float) -> np.ndarray:
    """Batch-norm followed by Eq. 1; ``bnp`` = (gamma, beta, mean, var)."""
    return sign(bn(x, *bnp, eps))
