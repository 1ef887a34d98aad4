"""GPU test aids around the parity tests: every entry point that writes a buffer is run
 * into an output that sits between sentinel words (nothing before or after it may change),
   once 16-byte aligned (vector stores) and once displaced by one element (scalar stores),
 * twice, into buffers that held different garbage (the two results must be identical: no
   read of uninitialised output, no order-dependent result),
and its integer / bit results are compared with the CPU oracle as in the parity tests.
Also here: flip words that carry set bits beyond the last column (they must not reach the
packed output), the headline 8192-cube compared with the oracle in full, and a large
convolution whose sizes are not powers of two."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1705_07175_amd import binding as esp
from paper_1705_07175_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
SENTINEL = {torch.int32: 0x5A5A5A5A, torch.int64: 0x5A5A5A5A5A5A5A5A, torch.float32: 12345.675, torch.uint8: 0x5A}
GARBAGE = {torch.int32: -0x12345678, torch.int64: -0x123456789ABCDEF, torch.float32: -7.25, torch.uint8: 0xC3}


@pytest.fixture(scope="module", autouse=True)
def _oracle_threads():
    oracle.set_threads(min(16, os.cpu_count() or 1))
    yield
    oracle.set_threads(1)


class Arena:
    """Hands out output buffers that lie between sentinel elements and checks them afterwards."""

    def __init__(self, guard, fill):
        self.guard, self.fill, self.bufs = guard, fill, []

    def __call__(self, shape, dtype, aligned=False):
        """aligned: this buffer must stay 16-byte aligned whatever the arena's guard (a workspace)."""
        n = int(np.prod(shape))
        guard = 64 if aligned else self.guard
        buf = torch.full((n + 2 * guard,), SENTINEL[dtype], dtype=dtype, device=DEV)
        view = buf[guard:guard + n]
        view.fill_(self.fill[dtype])
        self.bufs.append((buf, n, dtype, guard))
        return view.view(tuple(shape))

    def check(self, what):
        for i, (buf, n, dtype, guard) in enumerate(self.bufs):
            s = torch.tensor(SENTINEL[dtype], dtype=dtype, device=DEV)
            assert bool((buf[:guard] == s).all()), "%s: words before output %d were overwritten" % (what, i)
            assert bool((buf[guard + n:] == s).all()), "%s: words after output %d were overwritten" % (what, i)


def _pm1(seed, shape):
    return synth.pm1(np.random.default_rng(seed), shape)


def _dev_packed(pm1):
    return esp.to_packed_tensor(oracle.pack_bits(pm1), DEV)


def _f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def _fold(seed, n, scale):
    bnp = synth.bn_params(np.random.default_rng(seed), n)
    bnp = (bnp[0], bnp[1], (bnp[2] * scale).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    return bnp, torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV)


# Every case: fn(alloc) -> list of (device result, exact expected numpy array or None).
def case_pack(rows, k):
    def run(alloc):
        x = np.random.default_rng(rows + k).standard_normal((rows, k)).astype(np.float32)
        got = esp.pack_f32(_f32(x), out=alloc((rows, esp.words(k)), esp.PACKED))
        return [(got, oracle.pack_bits(oracle.sign(x)))]
    return run


def case_bgemm(M, N, K, mfma=False):
    def run(alloc):
        a, b = _pm1(M + N, (M, K)), _pm1(K, (N, K))
        fn = esp.bgemm_mfma if mfma else esp.bgemm
        got = fn(_dev_packed(a), _dev_packed(b), K, out=alloc((M, N), torch.int32))
        return [(got, oracle.dense_pm1(a, b))]
    return run


def case_unroll(B, H, W, C, kh, kw, stride, pad):
    def run(alloc):
        x = _pm1(B + H + C, (B, H, W, C))
        H2, W2 = esp.conv_out(H, kh, stride, pad), esp.conv_out(W, kw, stride, pad)
        got = esp.unroll(_dev_packed(x), C, kh, kw, stride, pad,
                         out=alloc((B * H2 * W2, kh * kw * esp.words(C)), esp.PACKED))
        rows = oracle.unroll_pm1(x, kh, kw, stride, pad, -1).reshape(B * H2 * W2, kh * kw, C)
        return [(got, oracle.pack_bits(rows).reshape(B * H2 * W2, -1))]
    return run


def case_bconv(B, H, W, C, L2, kh, kw, stride, pad, engine):
    def run(alloc):
        x, f = _pm1(B + C, (B, H, W, C)), _pm1(L2 + C, (L2, kh, kw, C))
        H2, W2 = esp.conv_out(H, kh, stride, pad), esp.conv_out(W, kw, stride, pad)
        ws = alloc((max(16, esp.bconv_workspace_bytes(B, H, W, C, kh, kw, stride, pad)),), torch.uint8, aligned=True)
        got = esp.bconv(_dev_packed(x), _dev_packed(f), C, stride, pad, workspace=ws,
                        out=alloc((B, H2, W2, L2), torch.int32), engine=engine)
        return [(got, oracle.conv_pm1(x, f, stride, pad, -1))]
    return run


def case_bn_sign_pack(rows, C, K):
    def run(alloc):
        rng = np.random.default_rng(rows + C)
        x = (rng.integers(-60, 61, size=(rows, C)) * 2 + (K % 2)).astype(np.int32)
        bnp, thr, flip = _fold(C, C, 1.0)
        got = esp.bn_sign_pack(torch.from_numpy(x).to(DEV), thr, flip, out=alloc((rows, esp.words(C)), esp.PACKED))
        return [(got, oracle.pack_bits(oracle.bn_sign(x, bnp, synth.BN_EPS)))]
    return run


def case_bgemm_bits(M, N, K, engine):
    def run(alloc):
        a, b = _pm1(M + N, (M, K)), _pm1(K, (N, K))
        bnp, thr, flip = _fold(N + K, N, np.sqrt(K))
        got = esp.bgemm_bn_sign_pack(_dev_packed(a), _dev_packed(b), K, thr, flip,
                                     out=alloc((M, esp.words(N)), esp.PACKED), engine=engine)
        return [(got, oracle.pack_bits(oracle.bn_sign(oracle.dense_pm1(a, b), bnp, synth.BN_EPS)))]
    return run


def case_bconv_bits(B, H, W, C, L2, kh, kw, stride, pad, engine, pool=False):
    def run(alloc):
        x, f = _pm1(B + C, (B, H, W, C)), _pm1(L2 + C, (L2, kh, kw, C))
        bnp, thr, flip = _fold(L2, L2, np.sqrt(kh * kw * C))
        H2, W2 = esp.conv_out(H, kh, stride, pad), esp.conv_out(W, kw, stride, pad)
        act = oracle.bn_sign(oracle.conv_pm1(x, f, stride, pad, -1), bnp, synth.BN_EPS)
        if pool:
            got = esp.bconv_bn_sign_pack_pool2(_dev_packed(x), _dev_packed(f), C, thr, flip, stride, pad,
                                               out=alloc((B, H2 // 2, W2 // 2, esp.words(L2)), esp.PACKED),
                                               engine=engine)
            return [(got, oracle.pack_bits(oracle.maxpool_pm1(act, 2, 2)))]
        ws = alloc((max(16, esp.bconv_workspace_bytes(B, H, W, C, kh, kw, stride, pad)),), torch.uint8, aligned=True)
        got = esp.bconv_bn_sign_pack(_dev_packed(x), _dev_packed(f), C, thr, flip, stride, pad, workspace=ws,
                                     out=alloc((B, H2, W2, esp.words(L2)), esp.PACKED), engine=engine)
        return [(got, oracle.pack_bits(act))]
    return run


def case_pad_correction(B, H, W, C, L2, kh, kw, stride, pad):
    def run(alloc):
        x, f = _pm1(B + C, (B, H, W, C)), _pm1(L2 + C, (L2, kh, kw, C))
        H2, W2 = esp.conv_out(H, kh, stride, pad), esp.conv_out(W, kw, stride, pad)
        fp = _dev_packed(f)
        corr = esp.pad_correction(fp, C, H, W, stride, pad, out=alloc((H2, W2, L2), torch.int32))
        out = esp.bconv(_dev_packed(x), fp, C, stride, pad, out=alloc((B, H2, W2, L2), torch.int32))
        esp.add_pad_correction(out, corr, H, W, kh, kw, stride, pad)     # in place, border pixels only
        return [(corr, oracle.conv_pm1(np.zeros((1, H, W, C), dtype=np.int8), f, stride, pad, +1)[0]),
                (out, oracle.conv_pm1(x, f, stride, pad, 0))]
    return run


def case_bmaxpool(B, H, W, C, win, stride):
    def run(alloc):
        x = np.where(np.random.default_rng(B + H).random((B, H, W, C)) < 0.25, 1, -1).astype(np.int8)
        H2, W2 = (H - win) // stride + 1, (W - win) // stride + 1
        got = esp.bmaxpool(_dev_packed(x), C, win, stride, out=alloc((B, H2, W2, esp.words(C)), esp.PACKED))
        return [(got, oracle.pack_bits(oracle.maxpool_pm1(x, win, stride)))]
    return run


def case_bitplane(M, N, K):
    def run(alloc):
        rng = np.random.default_rng(M + N + K)
        x = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
        w = synth.pm1(rng, (N, K))
        wp = _dev_packed(w)
        planes = esp.bitplane_pack_u8(torch.from_numpy(x).to(DEV), out=alloc((M, 8, esp.words(K)), esp.PACKED))
        want_planes = np.stack([oracle.pack_bits((((x >> i) & 1).astype(np.int8) * 2 - 1)) for i in range(8)], axis=1)
        wsum = esp.row_sums(wp, K, out=alloc((N,), torch.int32))
        d = esp.bgemm(planes.reshape(M * 8, -1), wp, K).reshape(M, 8, N)
        y = esp.bitplane_combine(d, wsum, out=alloc((M, N), torch.int32))
        want = oracle.dense_u8(x, w)
        bnp, thr, flip = _fold(N, N, 40 * np.sqrt(K))
        bits, y2 = esp.bitplane_dense(planes, wp, wsum, K, thr=thr, flip=flip,
                                      bits=alloc((M, esp.words(N)), esp.PACKED), y=alloc((M, N), torch.int32))
        return [(planes, want_planes), (wsum, w.astype(np.int64).sum(axis=1).astype(np.int32)), (y, want), (y2, want),
                (bits, oracle.pack_bits(oracle.bn_sign(want, bnp, synth.BN_EPS)))]
    return run


def _close_1e4(got, ref):
    assert np.all(np.abs(got.astype(np.float64) - ref) <= 1e-4 * np.maximum(1.0, np.abs(ref)))


def case_float_dense(M, N, K, packed_weights=False):
    # float outputs: closeness to the oracle here, bit-level rules in the parity tests; the sign bits
    # must be the exact decision on the kernel's own pre-activations
    def run(alloc):
        rng = np.random.default_rng(M + N + K)
        x = rng.random((M, K), dtype=np.float32)
        w = synth.pm1(rng, (N, K))
        bnp = synth.bn_params(rng, N)
        bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(K) + K / 4).astype(np.float32), bnp[3])
        thr, sgn = esp.bn_fold_f32(*bnp, synth.BN_EPS)
        thr_d, sgn_d = torch.from_numpy(thr).to(DEV), torch.from_numpy(sgn).to(DEV)
        ref = oracle.dense_f64(x, w)
        pre = alloc((M, N), torch.float32)
        if packed_weights:
            bits = esp.dense_f32_bw_bn_sign_pack(_f32(x), _dev_packed(w), thr_d, sgn_d,
                                                 out=alloc((M, esp.words(N)), esp.PACKED), pre=pre)
        else:
            bits = esp.dense_f32_bn_sign_pack(_f32(x), _f32(w), thr_d, sgn_d,
                                              out=alloc((M, esp.words(N)), esp.PACKED), pre=pre)
        _close_1e4(pre.cpu().numpy(), ref)
        own = oracle.pack_bits(oracle.bn_sign(pre.cpu().numpy(), bnp, synth.BN_EPS))
        res = [(bits, own), (pre, None)]
        if not packed_weights:
            y = esp.dense_f32(_f32(x), _f32(w), out=alloc((M, N), torch.float32))
            _close_1e4(y.cpu().numpy(), ref)
            again = esp.bn_sign_pack_f32(y, thr_d, sgn_d, out=alloc((M, esp.words(N)), esp.PACKED))
            res += [(y, None), (again, oracle.pack_bits(oracle.bn_sign(y.cpu().numpy(), bnp, synth.BN_EPS)))]
        return res
    return run


def case_float_conv(B, H, W, C, L2, k, stride, pad):
    def run(alloc):
        rng = np.random.default_rng(B + H + L2)
        x = rng.random((B, H, W, C), dtype=np.float32)
        f = synth.pm1(rng, (L2, k, k, C))
        bnp = synth.bn_params(rng, L2)
        thr, sgn = esp.bn_fold_f32(*bnp, synth.BN_EPS)
        H2, W2 = esp.conv_out(H, k, stride, pad), esp.conv_out(W, k, stride, pad)
        ref = oracle.conv_f64(x, f, stride, pad)
        y = esp.conv_f32(_f32(x), _f32(f), stride, pad, out=alloc((B, H2, W2, L2), torch.float32))
        _close_1e4(y.cpu().numpy(), ref)
        pre = alloc((B, H2, W2, L2), torch.float32)
        bits = esp.conv_f32_bn_sign_pack(_f32(x), _f32(f), torch.from_numpy(thr).to(DEV), torch.from_numpy(sgn).to(DEV),
                                         stride, pad, out=alloc((B, H2, W2, esp.words(L2)), esp.PACKED), pre=pre)
        _close_1e4(pre.cpu().numpy(), ref)
        return [(y, None), (pre, None), (bits, oracle.pack_bits(oracle.bn_sign(pre.cpu().numpy(), bnp, synth.BN_EPS)))]
    return run


CASES = {
    "pack_flat": case_pack(37, 1280), "pack_ragged": case_pack(5, 65),
    "bgemv": case_bgemm(1, 1000, 1024), "bgemv_8": case_bgemm(7, 2048, 1152),
    "bgemm_tile_32x64": case_bgemm(130, 70, 200), "bgemm_tile_k_tail": case_bgemm(300, 301, 8256),
    "bgemm_tile_128x64": case_bgemm(2100, 1990, 640), "bgemm_few_columns": case_bgemm(1024, 10, 1024),
    "bgemm_three_columns": case_bgemm(2000, 3, 70), "bgemm_mfma": case_bgemm(300, 200, 1000, mfma=True),
    "bgemm_mfma_big": case_bgemm(2000, 300, 1100, mfma=True),
    "unroll_vec": case_unroll(2, 7, 5, 256, 3, 3, 2, 1), "unroll_word": case_unroll(1, 6, 6, 100, 3, 3, 1, 1),
    "bconv_lowered": case_bconv(1, 6, 6, 100, 9, 3, 3, 1, 1, 0), "bconv_implicit": case_bconv(4, 16, 16, 128, 128, 3, 3, 1, 1, 0),
    "bconv_implicit_ragged": case_bconv(2, 9, 7, 256, 65, 5, 3, 2, 2, 0), "bconv_mfma": case_bconv(2, 9, 7, 256, 65, 5, 3, 2, 2, 1),
    "bn_sign_pack_ragged": case_bn_sign_pack(5, 70, 300), "bn_sign_pack_flat": case_bn_sign_pack(37, 1280, 2000),
    "bn_sign_pack_periodic": case_bn_sign_pack(1000, 128, 1152),
    "bits_gemv": case_bgemm_bits(2, 100, 70, 0), "bits_gemv_quarter_words": case_bgemm_bits(1, 1000, 4096, 0),
    "bits_few_rows": case_bgemm_bits(63, 9, 256, 0), "bits_tile_small": case_bgemm_bits(130, 70, 200, 0),
    "bits_tile_64": case_bgemm_bits(1000, 128, 1152, 0), "bits_tile_128x64": case_bgemm_bits(2100, 1990, 640, 0),
    "bits_mfma": case_bgemm_bits(130, 70, 200, 1), "bits_mfma_big": case_bgemm_bits(2100, 1990, 640, 1),
    "bconv_bits_lowered": case_bconv_bits(1, 6, 6, 100, 9, 3, 3, 1, 1, 0),
    "bconv_bits_few_rows": case_bconv_bits(2, 5, 5, 384, 64, 3, 3, 1, 1, 0),
    "bconv_bits_64": case_bconv_bits(8, 32, 32, 128, 128, 3, 3, 1, 1, 0),
    "bconv_bits_128x128": case_bconv_bits(40, 32, 32, 128, 256, 3, 3, 1, 1, 0),
    "bconv_bits_128x64_partial_word": case_bconv_bits(33, 32, 32, 128, 100, 3, 3, 1, 1, 0),
    "bconv_bits_mfma": case_bconv_bits(8, 32, 32, 128, 128, 3, 3, 1, 1, 1),
    "pool2_few_rows": case_bconv_bits(2, 8, 32, 128, 72, 3, 3, 1, 1, 0, pool=True),
    "pool2_tile": case_bconv_bits(5, 16, 16, 128, 100, 3, 3, 1, 1, 0, pool=True),
    "pool2_128": case_bconv_bits(40, 32, 32, 128, 256, 3, 3, 1, 1, 0, pool=True),
    "pool2_mfma": case_bconv_bits(5, 16, 16, 128, 100, 3, 3, 1, 1, 1, pool=True),
    "pad_correction": case_pad_correction(2, 5, 6, 128, 7, 3, 3, 1, 1),
    "pad_correction_scalar": case_pad_correction(2, 6, 7, 64, 6, 2, 2, 2, 1),
    "bmaxpool_vec": case_bmaxpool(2, 8, 8, 128, 2, 2), "bmaxpool_word": case_bmaxpool(2, 6, 6, 100, 3, 1),
    "bmaxpool_3_2": case_bmaxpool(3, 9, 11, 192, 3, 2),
    "bitplane": case_bitplane(3, 70, 200), "bitplane_big": case_bitplane(300, 257, 832),
    "float_dense_gemv": case_float_dense(3, 100, 50), "float_dense_mfma": case_float_dense(70, 130, 97),
    "float_dense_layer": case_float_dense(64, 4096, 784), "float_dense_packed_weights": case_float_dense(70, 130, 97, True),
    "float_dense_packed_weights_gemv": case_float_dense(2, 100, 50, True),
    "float_conv_general": case_float_conv(3, 9, 7, 3, 20, 3, 2, 1), "float_conv_3x3x3": case_float_conv(2, 32, 32, 3, 128, 3, 1, 1),
}


@pytest.mark.parametrize("guard", [64, 1], ids=["aligned", "displaced"])
@pytest.mark.parametrize("name", sorted(CASES))
def test_guard_words_and_run_twice(name, guard):
    """guard = 64 elements keeps every output 16-byte aligned (int32: 256 bytes, words: 512);
    guard = 1 displaces it by one element, which takes the narrower store paths."""
    first = Arena(guard, SENTINEL)
    res1 = CASES[name](first)
    torch.cuda.synchronize()
    first.check(name)
    second = Arena(guard, GARBAGE)
    res2 = CASES[name](second)
    torch.cuda.synchronize()
    second.check(name + " (second run)")
    assert len(res1) == len(res2)
    for i, ((g1, want), (g2, _)) in enumerate(zip(res1, res2)):
        assert torch.equal(g1, g2), "%s: output %d differs between two runs" % (name, i)
        if want is not None:
            got = g1.cpu().numpy()
            if g1.dtype == esp.PACKED:
                got = got.view(np.uint64)
            assert got.shape == want.shape, (name, i)
            assert np.array_equal(got, want), "%s: output %d differs from the oracle" % (name, i)


# ------------------------------------------------------------------------------ flip words with a dirty tail
def _dirty(flip, n):
    """The folded flip words with every bit beyond column n - 1 set."""
    f = esp.packed_to_numpy(flip).copy()
    if n % 64:
        f[-1] |= np.uint64(0xFFFFFFFFFFFFFFFF) << np.uint64(n % 64)
    return esp.to_packed_tensor(f, DEV)


@pytest.mark.parametrize("engine", [0, 1])
@pytest.mark.parametrize("M,N,K", [(2, 100, 70), (1, 1000, 4096), (8, 65, 1), (63, 9, 256), (200, 130, 1152),
                                   (130, 70, 200), (1000, 100, 1152), (2100, 1990, 640)])
def test_flip_bits_beyond_the_last_column_are_ignored_bgemm(M, N, K, engine):
    # Sec. 4.2 packing convention: tail bits of a packed row are zero, whatever the caller's flip word holds
    a, b = _pm1(M + N, (M, K)), _pm1(K, (N, K))
    bnp, thr, flip = _fold(N + K, N, np.sqrt(K))
    got = esp.bgemm_bn_sign_pack(_dev_packed(a), _dev_packed(b), K, thr, _dirty(flip, N), engine=engine)
    want = oracle.pack_bits(oracle.bn_sign(oracle.dense_pm1(a, b), bnp, synth.BN_EPS))
    assert np.array_equal(esp.packed_to_numpy(got), want)


def test_flip_bits_beyond_the_last_column_are_ignored_other_entry_points():
    rng = np.random.default_rng(5)
    for rows, C in ((5, 70), (40, 200)):
        x = (rng.integers(-60, 61, size=(rows, C)) * 2).astype(np.int32)
        bnp, thr, flip = _fold(C, C, 1.0)
        got = esp.bn_sign_pack(torch.from_numpy(x).to(DEV), thr, _dirty(flip, C))
        assert np.array_equal(esp.packed_to_numpy(got), oracle.pack_bits(oracle.bn_sign(x, bnp, synth.BN_EPS)))
    for engine in (0, 1):
        for (B, H, W, C, L2, pool) in ((33, 32, 32, 128, 100, False), (5, 16, 16, 128, 100, True),
                                        (2, 8, 32, 128, 72, True), (1, 6, 6, 100, 9, False)):
            x, f = _pm1(B + C, (B, H, W, C)), _pm1(L2 + C, (L2, 3, 3, C))
            bnp, thr, flip = _fold(L2, L2, np.sqrt(9 * C))
            act = oracle.bn_sign(oracle.conv_pm1(x, f, 1, 1, -1), bnp, synth.BN_EPS)
            if pool:
                got = esp.bconv_bn_sign_pack_pool2(_dev_packed(x), _dev_packed(f), C, thr, _dirty(flip, L2), 1, 1,
                                                   engine=engine)
                act = oracle.maxpool_pm1(act, 2, 2)
            else:
                got = esp.bconv_bn_sign_pack(_dev_packed(x), _dev_packed(f), C, thr, _dirty(flip, L2), 1, 1,
                                             engine=engine)
            assert np.array_equal(esp.packed_to_numpy(got), oracle.pack_bits(act)), (engine, B, L2, pool)
    # bit-plane dense layer (epilogue of the matrix-core kernel in plane mode)
    M, N, K = 33, 130, 1000
    xq = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    w = synth.pm1(rng, (N, K))
    wp = _dev_packed(w)
    bnp, thr, flip = _fold(N, N, 40 * np.sqrt(K))
    bits, _ = esp.bitplane_dense(esp.bitplane_pack_u8(torch.from_numpy(xq).to(DEV)), wp, esp.row_sums(wp, K), K,
                                 thr=thr, flip=_dirty(flip, N))
    assert np.array_equal(esp.packed_to_numpy(bits), oracle.pack_bits(oracle.bn_sign(oracle.dense_u8(xq, w), bnp, synth.BN_EPS)))


# ------------------------------------------------------------------------------ the headline product in full
@pytest.mark.parametrize("engine", ["xor_popcount", "mfma"])
def test_bgemm_config5_square_8192_in_full(engine):
    """All 67 108 864 outputs of the 8192-cube (Sec. 6.1, Table 1) against the oracle, in row blocks so
    that the oracle's progress is visible; the GPU result comes from ONE launch on the whole matrices."""
    n = 8192
    a, b = synth.config5_square(n)
    fn = esp.bgemm if engine == "xor_popcount" else esp.bgemm_mfma
    got = fn(esp.pack_f32(_f32(a)), esp.pack_f32(_f32(b)), n).cpu().numpy()
    step = 1024
    for r0 in range(0, n, step):
        want = oracle.dense_pm1(a[r0:r0 + step], b)
        assert np.array_equal(got[r0:r0 + step], want), "rows %d..%d" % (r0, r0 + step)
        print("8192-cube (%s): rows %d..%d identical" % (engine, r0, r0 + step), flush=True)


# ------------------------------------------------------------------------------ large implicit convolution, odd sizes
@pytest.mark.parametrize("engine", [0, 1])
def test_bconv_large_odd_sizes(engine):
    """Batch 64 of 31 x 31 x 128 -> 256 filters: 128 x 128 tiles whose row -> (image, y, x) split divides
    by 31 (no power of two anywhere), with a ragged last tile; int32 and thresholded outputs."""
    B, H, W, C, L2 = 64, 31, 31, 128, 256
    x, f = _pm1(1, (B, H, W, C)), _pm1(2, (L2, 3, 3, C))
    xp, fp = _dev_packed(x), _dev_packed(f)
    pre = oracle.conv_pm1(x, f, 1, 1, -1)
    assert np.array_equal(esp.bconv(xp, fp, C, 1, 1, engine=engine).cpu().numpy(), pre)
    bnp, thr, flip = _fold(3, L2, np.sqrt(9 * C))
    got = esp.bconv_bn_sign_pack(xp, fp, C, thr, flip, 1, 1, engine=engine)
    assert np.array_equal(esp.packed_to_numpy(got), oracle.pack_bits(oracle.bn_sign(pre, bnp, synth.BN_EPS)))
