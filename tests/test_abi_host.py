"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, rejects
bad arguments before touching the GPU, and its host-side batch-norm fold agrees with the
oracle's batch-norm + sign for every integer input (no GPU compute is called here)."""
import ctypes
import os
import re
import subprocess

import numpy as np
import pytest

import oracle
from paper_1705_07175_amd import binding as esp
from paper_1705_07175_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "espresso_hip.h")


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(esp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert "esp_bgemm" in names and "esp_bn_fold" in names and len(names) >= 13
    lib = esp.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(esp.EXPORTS)
    assert esp.version() >= 100
    assert esp.strerror(0) == "ESP_OK"
    assert "ESP_ESHAPE" in esp.strerror(-3)
    assert "unknown" in esp.strerror(-99)


def test_binding_prototypes_match_the_header():
    # every declared function has ctypes argument types of the declared arity and pointer-ness
    # (a missing prototype would pass 64-bit device pointers as 32-bit ints)
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    lib = esp.lib()
    seen = 0
    for m in re.finditer(r"\b(esp_[a-z0-9_]+)\s*\(([^)]*)\)\s*;", text):
        name, params = m.group(1), m.group(2).strip()
        plist = [] if params in ("", "void") else [q.strip() for q in params.split(",")]
        argtypes = getattr(lib, name).argtypes
        assert argtypes is not None and len(argtypes) == len(plist), name
        for decl, at in zip(plist, argtypes):
            is_ptr = "*" in decl or decl.startswith("esp_stream")
            assert is_ptr == (at in (ctypes.c_void_p, ctypes.c_char_p)), (name, decl, at)
            if "int64_t" in decl and not is_ptr:
                assert at is ctypes.c_int64, (name, decl)
            if "size_t" in decl and not is_ptr:
                assert at is ctypes.c_size_t, (name, decl)
        seen += 1
    assert seen == len(esp.EXPORTS)


def test_argument_errors_are_reported_without_a_gpu():
    lib = esp.lib()
    buf = (ctypes.c_uint64 * 64)()
    p = ctypes.addressof(buf)
    # null pointers / bad dimensions
    assert lib.esp_bgemm(None, p, p, 4, 4, 64, None) == -1
    assert lib.esp_bgemm(p, p, p, 4, 0, 64, None) == -1
    assert lib.esp_bgemm(p, p, p, -1, 4, 64, None) == -1
    assert lib.esp_bgemm(p, p, p, 4, 4, 1 << 30, None) == -3
    assert lib.esp_bgemm(p + 4, p, p, 4, 4, 64, None) == -2
    assert lib.esp_bgemm(None, None, None, 0, 4, 64, None) == 0        # empty M is a no-op
    assert lib.esp_bgemm_mfma(None, p, p, 4, 4, 64, None) == -1
    assert lib.esp_bgemm_mfma(p, p, p, 4, 4, 1 << 24, None) == -3
    assert lib.esp_pack_f32(None, p, 3, 64, None) == -1
    assert lib.esp_pack_f32(p, p + 4, 3, 64, None) == -2
    assert lib.esp_pack_f32(p, p, 0, 64, None) == 0
    assert lib.esp_pack_f32(p, p, 3, 0, None) == -1
    assert lib.esp_unroll(p, p, 1, 4, 4, 64, 7, 3, 1, 1, None) == -3    # kernel larger than padded input
    assert lib.esp_unroll(p, p, 1, 4, 4, 64, 3, 3, 0, 1, None) == -3    # stride < 1
    assert lib.esp_unroll(p, p, 1, 4, 4, 64, 3, 3, 1, -1, None) == -3   # pad < 0
    assert lib.esp_unroll(None, p, 1, 4, 4, 64, 3, 3, 1, 1, None) == -1
    assert lib.esp_bconv(p, p, p, 1, 4, 4, 64, 8, 3, 3, 1, 1, None, 0, None) == -4
    assert lib.esp_bconv_mfma(p, p, p, 1, 4, 4, 64, 8, 3, 3, 1, 1, None, 0, None) == -4
    assert lib.esp_bconv_bn_sign_pack(p, p, p, p, p, 1, 4, 4, 64, 8, 3, 3, 1, 1, p, 1 << 20, 7, None) == -1
    assert lib.esp_bgemm_bn_sign_pack(p, p, p, p, p, 4, 4, 64, 3, None) == -1
    assert lib.esp_bconv(p, p, p, 1, 4, 4, 64, 8, 3, 3, 1, 1, p, 8, None) == -4
    assert lib.esp_bconv_workspace_bytes(2, 4, 4, 64, 3, 3, 1, 1) == 2 * 16 * 9 * 8
    assert lib.esp_bconv_workspace_bytes(2, 4, 4, 65, 3, 3, 1, 1) == 2 * 16 * 9 * 16
    assert lib.esp_bconv_workspace_bytes(2, 4, 4, 64, 7, 3, 1, 1) == 0
    assert lib.esp_bmaxpool(p, p, 1, 4, 4, 64, 5, 2, None) == -3        # pooled size 0
    assert lib.esp_bmaxpool(p, p, 1, 4, 4, 64, 2, 0, None) == -3
    assert lib.esp_dense_f32_bw_bn_sign_pack(p, None, p, p, p, None, 1, 64, 64, None) == -1
    assert lib.esp_dense_f32_bw_bn_sign_pack(p, p + 4, p, p, p, None, 1, 64, 64, None) == -2
    assert lib.esp_dense_f32_bw_bn_sign_pack(p, p, p, p, p, None, 1, 64, 1 << 30, None) == -3
    assert lib.esp_dense_f32_bw_bn_sign_pack(None, None, None, None, None, None, 0, 64, 64, None) == 0
    # sizes beyond what the kernels' 32-bit piece and tile indices hold are refused, not launched
    assert lib.esp_unroll(p, p, 65536, 64, 64, 128, 3, 3, 1, 1, None) == -3
    assert lib.esp_bmaxpool(p, p, 1 << 20, 64, 64, 128, 2, 2, None) == -3
    assert lib.esp_bgemm(p, p, p, 1 << 31, 4, 64, None) == -3
    assert lib.esp_bgemm(p, p, p, 1 << 22, 1 << 22, 64, None) == -3     # more than 2^30 tiles
    assert lib.esp_bn_sign_pack(p, p, None, p, 4, 64, None) == -1
    assert lib.esp_bn_sign_pack(p, p, p, p, 4, 0, None) == -1
    assert lib.esp_dense_f32(p, None, p, 4, 4, 4, None) == -1
    assert lib.esp_conv_f32(p, p, p, 1, 4, 4, 3, 8, 3, 3, 0, 1, None) == -3
    assert lib.esp_bn_sign_pack_f32(p, p, None, p, 4, 64, None) == -1
    assert lib.esp_bn_fold_f32(p, p, p, None, 1e-4, 4, p, p) == -1
    assert lib.esp_pad_correction(p, None, 4, 4, 64, 8, 3, 3, 1, 1, None) == -1
    assert lib.esp_pad_correction(p, p, 4, 4, 64, 8, 7, 3, 1, 1, None) == -3
    assert lib.esp_add_pad_correction(None, p, 1, 4, 4, 8, 3, 3, 1, 1, None) == -1
    assert lib.esp_add_pad_correction(p, p, 0, 4, 4, 8, 3, 3, 1, 1, None) == 0
    assert lib.esp_bitplane_pack_u8(p, None, 2, 1, 64, None) == -1
    assert lib.esp_bitplane_pack_u8(p, p, 2, 1, 1 << 22, None) == -3
    assert lib.esp_row_sums(None, p, 4, 1, 64, None) == -1
    assert lib.esp_row_sums(p, p, 4, 1, 65, None) == -3
    assert lib.esp_bitplane_combine(p, p, None, 2, 1, 4, None) == -1
    assert lib.esp_conv_f32_bn_sign_pack(p, p, p, p, None, None, 1, 4, 4, 3, 8, 3, 3, 1, 1, None) == -1
    assert lib.esp_bn_fold(None, p, p, p, 1e-4, 4, p, p) == -1
    assert lib.esp_dense_f32_bn_sign_pack(p, p, p, None, p, None, 1, 4, 4, None) == -1
    assert lib.esp_dense_f32_bn_sign_pack(p, p, p, p, p + 4, None, 1, 4, 4, None) == -2
    assert lib.esp_dense_f32_bn_sign_pack(p, p, p, p, p, None, 0, 4, 4, None) == 0
    assert lib.esp_xor_popcount_probe(p, 4, 4, 0, None, None) == -1
    # the convolution that brings its own scratch: argument errors as esp_bconv, no GPU call is reached
    assert lib.esp_bconv_noalloc(p, p, None, 1, 4, 4, 64, 8, 3, 3, 1, 1, None) == -1
    assert lib.esp_bconv_noalloc(None, p, p, 1, 4, 4, 64, 8, 3, 3, 1, 1, None) == -1
    assert lib.esp_bconv_noalloc(p, p, p, 1, 4, 4, 64, 8, 7, 3, 1, 1, None) == -3
    assert lib.esp_bconv_noalloc(p, p, p, 1, 4, 4, 64, 8, 3, 3, 0, 1, None) == -3
    assert lib.esp_bconv_noalloc(p, p, p, 0, 4, 4, 64, 8, 3, 3, 1, 1, None) == 0
    assert lib.esp_bconv_noalloc(p, p, p, 256, 32, 32, 64, 8, 3, 3, 1, 1, None) == -4      # 18 MiB > 16 MiB
    assert lib.esp_bitplane_dense(p, p, p, None, None, None, None, 2, 64, 64, None) == -1
    assert lib.esp_bitplane_dense(p, p, p, None, None, p, None, 2, 64, 64, None) == -1
    assert lib.esp_bitplane_dense(p, p, p, p, p, p, p, 2, 64, 1 << 21, None) == -3
    assert lib.esp_bitplane_dense(p, p, p, p, p, p, p, 0, 64, 64, None) == 0
    assert lib.esp_bitplane_dense(p, p, p + 2, p, p, p, p, 2, 64, 64, None) == -2
    assert lib.esp_xor_popcount_probe(p, 0, 4, 0, p, None) == -1
    assert lib.esp_xor_popcount_probe(p, 4, 4, 3, p, None) == -1
    assert lib.esp_xor_popcount_probe(p, 4, (1 << 20) + 1, 2, p, None) == -3
    # fused pool: shapes that cannot hold whole row pairs in a tile are refused up front
    assert lib.esp_bconv_pool2_fusable(32, 32, 128, 3, 3, 1, 1) == 1
    assert lib.esp_bconv_pool2_fusable(8, 8, 512, 3, 3, 1, 1) == 1
    assert lib.esp_bconv_pool2_fusable(32, 32, 64, 3, 3, 1, 1) == 0
    assert lib.esp_bconv_pool2_fusable(7, 8, 128, 3, 3, 1, 1) == 0
    assert lib.esp_bconv_pool2_fusable(8, 12, 128, 3, 3, 1, 1) == 0
    assert lib.esp_bconv_pool2_fusable(8, 128, 128, 3, 3, 1, 1) == 0
    assert lib.esp_bconv_pool2_fusable(8, 8, 128, 3, 3, 0, 1) == 0
    assert lib.esp_bconv_bn_sign_pack_pool2(p, p, p, p, None, 1, 8, 8, 128, 8, 3, 3, 1, 1, 0, None) == -1
    assert lib.esp_bconv_bn_sign_pack_pool2(p, p, p, p, p, 1, 8, 8, 128, 8, 3, 3, 1, 1, 5, None) == -1
    assert lib.esp_bconv_bn_sign_pack_pool2(p, p, p, p, p, 1, 8, 8, 64, 8, 3, 3, 1, 1, 0, None) == -3
    assert lib.esp_bconv_bn_sign_pack_pool2(p, p, p, p, p, 1, 7, 8, 128, 8, 3, 3, 1, 1, 0, None) == -3
    assert lib.esp_bconv_bn_sign_pack_pool2(p + 8, p, p, p, p, 1, 8, 8, 128, 8, 3, 3, 1, 1, 0, None) == -2
    assert lib.esp_bconv_bn_sign_pack_pool2(p, p, p, p, p, 0, 8, 8, 128, 8, 3, 3, 1, 1, 0, None) == 0


def test_empty_batches_are_no_ops_without_a_gpu():
    # a zero batch / zero rows returns ESP_OK before anything is launched (no GPU here)
    lib = esp.lib()
    buf = (ctypes.c_uint64 * 64)()
    p = ctypes.addressof(buf)
    assert lib.esp_unroll(p, p, 0, 4, 4, 64, 3, 3, 1, 1, None) == 0
    assert lib.esp_bconv(p, p, p, 0, 4, 4, 64, 8, 3, 3, 1, 1, None, 0, None) == 0
    assert lib.esp_bconv_mfma(p, p, p, 0, 4, 4, 64, 8, 3, 3, 1, 1, None, 0, None) == 0
    assert lib.esp_bconv_bn_sign_pack(p, p, p, p, p, 0, 4, 4, 64, 8, 3, 3, 1, 1, None, 0, 0, None) == 0
    assert lib.esp_bgemm_bn_sign_pack(p, p, p, p, p, 0, 4, 64, 2, None) == 0
    assert lib.esp_bgemm_mfma(p, p, p, 0, 4, 64, None) == 0
    assert lib.esp_bmaxpool(p, p, 0, 4, 4, 64, 2, 2, None) == 0
    assert lib.esp_bn_sign_pack(p, p, p, p, 0, 64, None) == 0
    assert lib.esp_bn_sign_pack_f32(p, p, p, p, 0, 64, None) == 0
    assert lib.esp_dense_f32(p, p, p, 0, 4, 4, None) == 0
    assert lib.esp_conv_f32(p, p, p, 0, 4, 4, 3, 8, 3, 3, 1, 1, None) == 0
    assert lib.esp_conv_f32_bn_sign_pack(p, p, p, p, p, None, 0, 4, 4, 3, 8, 3, 3, 1, 1, None) == 0
    assert lib.esp_bitplane_pack_u8(p, p, 0, 1, 64, None) == 0
    assert lib.esp_bitplane_combine(p, p, p, 0, 1, 4, None) == 0


def _check_fold(gamma, beta, mean, var, eps, lo, hi):
    thr, flip = esp.bn_fold(gamma, beta, mean, var, eps)
    C = len(gamma)
    xs = np.arange(lo, hi + 1, dtype=np.int32)
    x = np.repeat(xs[:, None], C, axis=1)
    want = oracle.sign(oracle.bn(x, gamma, beta, mean, var, eps)) > 0
    flipbits = np.array([(int(flip[c // 64]) >> (c % 64)) & 1 for c in range(C)], dtype=bool)
    got = (x >= thr[None, :]) ^ flipbits[None, :]
    bad = np.argwhere(got != want)
    assert bad.size == 0, (bad[:5], thr, flipbits)
    return thr, flipbits


def test_bn_fold_exhaustive_random_channels():
    # every integer in [-K, K] for the largest K of the paper's networks (3*3*512 = 4608),
    # parameters drawn as for the benchmark configurations (about half the gammas negative)
    rng = np.random.default_rng(7)
    g, b, m, v = synth.bn_params(rng, 192)
    _check_fold(g, b, m, v, synth.BN_EPS, -4608, 4608)


def test_bn_fold_crafted_channels():
    g = np.array([1.0, -1.0, 0.0, 0.0, 2.0, -3.0, 1e-30, -1e-30, 1.0, -1.0, 1.0, 5.0], dtype=np.float32)
    b = np.array([0.0, 0.0, 0.5, -0.5, 1e10, 1e10, 0.0, 0.0, -3.0, -3.0, 0.0, -1e10], dtype=np.float32)
    m = np.array([3.0, 3.0, 0.0, 0.0, 0.0, 0.0, 2.0, 2.0, 0.5, 0.5, -7.0, 0.0], dtype=np.float32)
    v = np.array([0.75, 0.75, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 0.75, 0.75, 3.75, 1.0], dtype=np.float32)
    thr, flipbits = _check_fold(g, b, m, v, 0.25, -300, 300)
    # exact ties y(x) == 0 give +1: gamma=1, beta=0, mean=3 -> bit set from x = 3 on
    assert thr[0] == 3 and not flipbits[0]
    # gamma=-1: non-negative up to x = 3, so bit = NOT(x >= 4)
    assert thr[1] == 4 and flipbits[1]
    # gamma == 0: constant sign(beta)
    assert not flipbits[2] and flipbits[3] and thr[2] == thr[3] == np.iinfo(np.int32).min
    # |beta| so large that the bit never changes over the legal range
    assert not flipbits[4] and thr[4] == np.iinfo(np.int32).min
    assert thr[5] == np.iinfo(np.int32).min
    assert flipbits[11]
    # mean = -7, beta = 0: threshold -7
    assert thr[10] == -7


def test_bn_fold_tail_channels_and_flip_words():
    rng = np.random.default_rng(8)
    g, b, m, v = synth.bn_params(rng, 70)
    thr, flip = esp.bn_fold(g, b, m, v, 1e-4)
    assert thr.shape == (70,) and flip.shape == (2,)
    assert int(flip[1]) >> 6 == 0      # bits above channel 69 stay clear


def test_bn_fold_f32_matches_oracle_around_every_threshold():
    # the float fold must reproduce sign(batch-norm(x)) for every float x: check a dense set of
    # floats around each channel's threshold, plus zeros, extremes and random values
    rng = np.random.default_rng(9)
    C = 96
    g, b, m, v = synth.bn_params(rng, C)
    g[:4] = [0.0, 0.0, 1e-30, -1e-30]
    b[:4] = [0.5, -0.5, 1.0, -1.0]
    g[4:8] = [1.0, -1.0, 2.0, -3.0]
    b[4:8] = [1e30, 1e30, -1e30, -1e30]          # never / always flips within finite floats
    thr, sgn = esp.bn_fold_f32(g, b, m, v, synth.BN_EPS)
    assert set(np.unique(sgn)) <= {-1.0, 1.0}
    cols = []
    t = np.where(np.isfinite(thr), sgn * thr, 0.0).astype(np.float32)
    lo, hi = t.copy(), t.copy()
    cols.append(t.copy())
    for _ in range(40):
        lo = np.nextafter(lo, np.float32(-np.inf))
        hi = np.nextafter(hi, np.float32(np.inf))
        cols += [lo.copy(), hi.copy()]
    fmax = np.finfo(np.float32).max
    for val in (0.0, -0.0, fmax, -fmax, 1e-45, -1e-45):
        cols.append(np.full(C, val, dtype=np.float32))
    cols += list((rng.standard_normal((200, C)) * 50).astype(np.float32))
    x = np.stack(cols)
    want = oracle.sign(oracle.bn(x.astype(np.float64), g, b, m, v, synth.BN_EPS)) > 0
    got = (sgn[None, :] * x) >= thr[None, :]
    assert np.array_equal(got, want)


_SANITIZER_MAIN = r"""
// Drives the library's host code (status strings, both batch-norm folds) under AddressSanitizer and
// UndefinedBehaviorSanitizer.  stdin: C, eps, then gamma / beta / mean / var (C floats each) as text;
// stdout: thr flipbit (integer fold), then thr sgn as hex floats (float fold), one channel per line.
#include <cstdio>
#include <cstdint>
#include <vector>
#include "espresso_hip.h"
int main()
{
    int C;
    float eps;
    if (std::scanf("%d %f", &C, &eps) != 2) return 2;
    std::vector<float> p[4];
    for (auto &v : p) { v.resize(C); for (int c = 0; c < C; ++c) if (std::scanf("%f", &v[c]) != 1) return 2; }
    // exactly sized outputs: a write past either end is an error report
    std::vector<int32_t> thr(C);
    std::vector<uint64_t> flip((C + 63) / 64);
    if (esp_bn_fold(p[0].data(), p[1].data(), p[2].data(), p[3].data(), eps, C, thr.data(), flip.data()) != ESP_OK) return 3;
    std::vector<float> thrf(C), sgn(C);
    if (esp_bn_fold_f32(p[0].data(), p[1].data(), p[2].data(), p[3].data(), eps, C, thrf.data(), sgn.data()) != ESP_OK) return 4;
    for (int c = 0; c < C; ++c) std::printf("%d %d\n", thr[c], (int)((flip[c / 64] >> (c % 64)) & 1));
    for (int c = 0; c < C; ++c) std::printf("%a %a\n", thrf[c], sgn[c]);
    for (int st = -8; st <= 1; ++st) if (!esp_strerror(st)) return 5;
    if (esp_bn_fold(nullptr, p[1].data(), p[2].data(), p[3].data(), eps, C, thr.data(), flip.data()) != ESP_EINVAL) return 6;
    if (esp_bn_fold(p[0].data(), p[1].data(), p[2].data(), p[3].data(), eps, 0, thr.data(), flip.data()) == ESP_OK) return 7;
    return 0;
}
"""


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """csrc/host.cpp built on the side with -fsanitize=address,undefined (CPU only; the GPU sources are not
    part of it) and run on crafted + random channels, 70 of them so that the last flip word is partial: no
    sanitizer report, and the folds it prints are the ones the product library computes."""
    main = tmp_path / "san_main.cpp"
    main.write_text(_SANITIZER_MAIN)
    exe = tmp_path / "san_host"
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    subprocess.run(["g++", "-O1", "-g", "-std=c++17", "-ffp-contract=off", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
                    "-I", os.path.join(root, "include"), str(main),
                    os.path.join(root, "paper_1705_07175_amd", "csrc", "host.cpp"), "-o", str(exe)], check=True)
    rng = np.random.default_rng(12)
    C = 70
    g, b, m, v = synth.bn_params(rng, C)
    g[:8] = [0.0, 0.0, 1e-30, -1e-30, 1.0, -1.0, 2.0, -3.0]
    b[:8] = [0.5, -0.5, 1.0, -1.0, 1e30, 1e30, -1e30, -1e30]
    m[8:12] = [3e9, -3e9, 0.0, 1e-20]
    text = "%d %r\n" % (C, float(synth.BN_EPS)) + "\n".join(" ".join(repr(float(x)) for x in a) for a in (g, b, m, v)) + "\n"
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([str(exe)], input=text, env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True)
    assert r.returncode == 0, (r.returncode, r.stderr[-2000:])
    assert "runtime error" not in r.stderr and "Sanitizer" not in r.stderr, r.stderr[-2000:]
    lines = r.stdout.split("\n")
    thr, flip = esp.bn_fold(g, b, m, v, synth.BN_EPS)
    for c in range(C):
        t, f = lines[c].split()
        assert int(t) == int(thr[c]) and int(f) == (int(flip[c // 64]) >> (c % 64)) & 1, c
    thrf, sgn = esp.bn_fold_f32(g, b, m, v, synth.BN_EPS)
    for c in range(C):
        t, sg = lines[C + c].split()
        assert float.fromhex(t) == float(thrf[c]) and float.fromhex(sg) == float(sgn[c]), c


def test_bench_refuses_more_than_one_gpu():
    # one GPU only: the benchmark says so and exits before touching any device
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120)
    assert res.returncode != 0 and "ONE GPU" in res.stderr and res.stdout.strip() == ""
