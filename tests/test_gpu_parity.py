"""GPU parity: every C-ABI entry point against the CPU oracle, element by element, on the
same seeded inputs.  Integer, bit and index results must be identical; the float first
layer is held to 1e-4 relative on pre-activations (see the float tests)."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1705_07175_amd import binding as esp
from paper_1705_07175_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"


@pytest.fixture(scope="module", autouse=True)
def _oracle_threads():
    oracle.set_threads(min(16, os.cpu_count() or 1))
    yield
    oracle.set_threads(1)


def _pm1(rng, shape):
    return synth.pm1(rng, shape)


def _f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def _packed_dev(pm1):
    """+-1 int8 array -> packed device tensor, packed by the ORACLE (so that bgemm, unroll, ...
    are tested independently of the GPU pack kernel)."""
    return esp.to_packed_tensor(oracle.pack_bits(pm1), DEV)


# ------------------------------------------------------------------------------ pack
@pytest.mark.parametrize("rows,k", [(1, 1), (1, 64), (3, 63), (5, 65), (17, 200), (64, 1024),
                                    (1000, 1000), (33, 4096), (2500, 128), (1, 16384), (37, 1280), (9, 1088),
                                    (5, 192), (3, 64)])
def test_pack_f32(rows, k):
    rng = np.random.default_rng(rows * 100003 + k)
    x = rng.standard_normal((rows, k)).astype(np.float32)
    x[rng.random((rows, k)) < 0.05] = 0.0
    x[rng.random((rows, k)) < 0.05] = -0.0
    got = esp.packed_to_numpy(esp.pack_f32(_f32(x)))
    want = oracle.pack_bits(oracle.sign(x))
    assert got.shape == want.shape
    assert np.array_equal(got, want)


def test_pack_f32_special_values_and_nhwc():
    x = np.array([[0.0, -0.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 5.0]], dtype=np.float32)
    got = esp.packed_to_numpy(esp.pack_f32(_f32(x)))
    assert int(got[0, 0]) == 0b10101011
    rng = np.random.default_rng(1)
    t = _pm1(rng, (2, 5, 7, 130))
    got = esp.packed_to_numpy(esp.pack_f32(_f32(t)))
    assert got.shape == (2, 5, 7, 3)
    assert np.array_equal(got, oracle.pack_bits(t))


def test_pack_f32_empty():
    out = esp.pack_f32(torch.empty((0, 128), dtype=torch.float32, device=DEV))
    assert out.shape == (0, 2)


# ------------------------------------------------------------------------------ bgemm
BGEMM_SHAPES = [
    (1, 1, 64), (2, 3, 128), (3, 2, 192), (9, 5, 7), (16, 16, 65),           # tiny, tails
    (1, 1000, 1024), (1, 77, 64), (2, 130, 200), (3, 64, 16384), (4, 513, 4096),
    (5, 33, 100), (7, 2048, 1152), (8, 10, 4096), (1, 10, 1024),             # small-M kernel
    (9, 10, 4096), (64, 1024, 1024), (130, 70, 200), (257, 513, 1152),       # 64x64 tiles
    (100, 1000, 64), (65, 129, 4608), (1024, 10, 1024), (300, 301, 8256),
    (1024, 10, 4096), (100, 16, 200), (9, 1, 64), (300, 8, 8256), (64, 9, 8192), (2000, 3, 70),   # few columns
    (33, 17, 128), (3, 5, 1), (70, 70, 1),                                      # a single bit per row
]


@pytest.mark.parametrize("M,N,K", BGEMM_SHAPES)
def test_bgemm(M, N, K):
    rng = np.random.default_rng(M * 7919 + N * 104729 + K)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    got = esp.bgemm(_packed_dev(a), _packed_dev(b), K).cpu().numpy()
    assert np.array_equal(got, oracle.dense_pm1(a, b))


@pytest.mark.parametrize("M,N,K", BGEMM_SHAPES + [(256, 128, 512), (300, 200, 1000), (513, 130, 4160)])
def test_bgemm_mfma(M, N, K):
    rng = np.random.default_rng(M * 7919 + N * 104729 + K + 1)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    got = esp.bgemm_mfma(_packed_dev(a), _packed_dev(b), K).cpu().numpy()
    assert np.array_equal(got, oracle.dense_pm1(a, b))


# the matrix-core kernel checked in full against the oracle on large products with ragged edges
# (thousands of 256 x 128 blocks, many tile rows per XCD group, a very tall and narrow product);
# int32 and thresholded outputs
@pytest.mark.parametrize("M,N,K", [(4100, 4100, 200), (131072 + 70, 100, 192), (2000, 300, 1100)])
def test_bgemm_mfma_block_shapes(M, N, K):
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    want = oracle.dense_pm1(a, b)
    ap, bp = _packed_dev(a), _packed_dev(b)
    got = esp.bgemm_mfma(ap, bp, K)
    assert np.array_equal(got.cpu().numpy(), want)
    del got
    bnp = synth.bn_params(rng, N)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(K)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    bits = esp.bgemm_bn_sign_pack(ap, bp, K, torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV),
                                  engine=esp.ENGINE_MFMA)
    assert np.array_equal(esp.packed_to_numpy(bits), oracle.pack_bits(oracle.bn_sign(want, bnp, synth.BN_EPS)))


@pytest.mark.parametrize("n", [2048, 8192])
def test_bgemm_mfma_config5_square_sampled(n):
    a, b = synth.config5_square(n)
    c = esp.bgemm_mfma(_packed_dev(a), _packed_dev(b), n).cpu().numpy()
    _check_sampled(a, b, c, np.random.default_rng(n + 1))


def test_bgemm_config1():
    a, b = synth.config1()
    got = esp.bgemm(_packed_dev(a), _packed_dev(b), 1024).cpu().numpy()
    assert got.shape == (64, 1024)
    assert np.array_equal(got, oracle.dense_pm1(a, b))


def test_bgemm_large_tile_path_full():
    # enough tiles for the large-tile kernel (128x64 on packed matrices), ragged in M and N, several K stages
    M, N, K = 2900, 2950, 2240
    rng = np.random.default_rng(5)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    got = esp.bgemm(_packed_dev(a), _packed_dev(b), K).cpu().numpy()
    assert np.array_equal(got, oracle.dense_pm1(a, b))


# every length of the last K stage (1 to 8 k-groups of 128 bits, handled two at a time with an odd
# one at the end), an odd number of words per row (8-byte loads) and a K that is not a multiple of
# 64, on each tile shape a packed-matrix product can take (32x64, 64x64, 128x64; 128x128 serves
# convolutions and is covered by the fused convolution cases)
@pytest.mark.parametrize("M,N,Ks", [
    (130, 70, (1088, 1152, 1280, 1344, 1472, 1600, 1728, 1856, 1984, 2048, 2112, 1100, 960, 64)),
    (1100, 1100, (1152, 1280, 1472, 1728, 1984, 2112, 1100)),
    (2100, 1990, (1152, 1344, 1600, 2112, 1100, 64)),
    (2900, 2950, (1152, 1344, 1600, 2112)),
])
def test_bgemm_tile_k_tails(M, N, Ks):
    for K in Ks:
        rng = np.random.default_rng(M + 31 * K)
        a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
        got = esp.bgemm(_packed_dev(a), _packed_dev(b), K).cpu().numpy()
        assert np.array_equal(got, oracle.dense_pm1(a, b)), K


def _check_sampled(a, b, c, rng, nrows=6, ncols=6):
    """Sampled rows and columns bit-exact plus the full-matrix checksum identities
    sum_n C[m][n] = a_m . (sum_n b_n) and its column analogue, which touch every output."""
    M, K = a.shape
    N = b.shape[0]
    rows = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, nrows)]))
    cols = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, ncols)]))
    assert np.array_equal(c[rows], oracle.dense_pm1(a[rows], b))
    assert np.array_equal(c[:, cols], oracle.dense_pm1(a, b[cols]))
    bsum = b.astype(np.int64).sum(axis=0)
    asum = a.astype(np.int64).sum(axis=0)
    assert np.array_equal(c.sum(axis=1, dtype=np.int64), a.astype(np.int64) @ bsum)
    assert np.array_equal(c.sum(axis=0, dtype=np.int64), b.astype(np.int64) @ asum)


@pytest.mark.parametrize("n", [2048, 4096, 8192])
def test_bgemm_config5_square_sampled(n):
    a, b = synth.config5_square(n)
    c = esp.bgemm(_packed_dev(a), _packed_dev(b), n).cpu().numpy()
    _check_sampled(a, b, c, np.random.default_rng(n))


def test_bgemm_config5_gemv():
    a, b = synth.config5_gemv()
    c = esp.bgemm(_packed_dev(a), _packed_dev(b), 16384).cpu().numpy()
    assert c.shape == (1, 16384)
    assert np.array_equal(c, oracle.dense_pm1(a, b))


def test_bgemm_closed_forms_on_gpu():
    K = 1000
    rng = np.random.default_rng(9)
    a = _pm1(rng, (40, K))
    ap = _packed_dev(a)
    c = esp.bgemm(ap, ap, K).cpu().numpy()
    assert np.all(np.diag(c) == K) and np.array_equal(c, c.T)
    c = esp.bgemm(ap, _packed_dev(-a), K).cpu().numpy()
    assert np.all(np.diag(c) == -K)


@pytest.mark.parametrize("M", [1, 9])
def test_bgemm_longest_rows_closed_forms(M):
    # the longest legal rows (K = 2^30 - 64: 128 MiB per packed row); the oracle's unpacked
    # operands would not fit, so the expected values are closed forms: equal rows give +K,
    # complementary rows -K, one differing word K - 128 (the int32 contract at its edge)
    K = (1 << 30) - 64
    Kw = K // 64
    a = torch.full((M, Kw), -1, dtype=esp.PACKED, device=DEV)          # all +1
    b = torch.full((3, Kw), -1, dtype=esp.PACKED, device=DEV)
    b[1].zero_()                                                       # all -1
    b[2, Kw // 2] = 0                                                  # 64 values differ
    c = esp.bgemm(a, b, K).cpu().numpy()
    assert np.array_equal(c, np.tile(np.array([K, -K, K - 128], dtype=np.int32), (M, 1)))
    lib_status = esp.lib().esp_bgemm(a.data_ptr(), b.data_ptr(), a.data_ptr(), M, 3, 1 << 30, None)
    assert lib_status == -3                                            # K = 2^30 is refused


def test_bgemm_mfma_longest_rows_closed_forms():
    K = (1 << 24) - 64                                                 # fp32-exact accumulation limit
    Kw = K // 64
    a = torch.full((9, Kw), -1, dtype=esp.PACKED, device=DEV)
    a[3].zero_()
    b = torch.full((3, Kw), -1, dtype=esp.PACKED, device=DEV)
    b[1].zero_()
    b[2, 7] = 0
    want = np.tile(np.array([K, -K, K - 128], dtype=np.int32), (9, 1))
    want[3] = [-K, K, -(K - 128)]
    assert np.array_equal(esp.bgemm_mfma(a, b, K).cpu().numpy(), want)
    assert np.array_equal(esp.bgemm(a, b, K).cpu().numpy(), want)


def test_bgemm_unaligned_views():
    # rows of odd word count and a base pointer that is only 8-byte aligned
    M, N, K = 20, 30, 192
    rng = np.random.default_rng(10)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    abuf = torch.zeros(M * 3 + 1, dtype=esp.PACKED, device=DEV)
    bbuf = torch.zeros(N * 3 + 1, dtype=esp.PACKED, device=DEV)
    av = abuf[1:].view(M, 3)
    bv = bbuf[1:].view(N, 3)
    av.copy_(_packed_dev(a))
    bv.copy_(_packed_dev(b))
    cbuf = torch.zeros(M * N + 1, dtype=torch.int32, device=DEV)
    cv = cbuf[1:].view(M, N)
    esp.bgemm(av, bv, K, out=cv)
    assert np.array_equal(cv.cpu().numpy(), oracle.dense_pm1(a, b))
    assert int(cbuf[0]) == 0


# ------------------------------------------------------------------------------ unroll / bconv
CONV_CASES = [
    # B, H, W, C, L2, kh, kw, stride, pad
    (1, 4, 4, 64, 3, 3, 3, 1, 1),
    (2, 5, 6, 128, 7, 3, 3, 1, 1),
    (2, 7, 5, 192, 5, 3, 3, 2, 1),
    (1, 6, 6, 100, 9, 3, 3, 1, 1),       # channel tail inside every tap
    (3, 8, 8, 64, 130, 1, 1, 1, 0),
    (2, 9, 7, 256, 65, 5, 3, 2, 2),
    (1, 8, 8, 512, 70, 3, 3, 1, 1),
    (2, 6, 6, 128, 16, 2, 2, 2, 0),
    (4, 16, 16, 128, 128, 3, 3, 1, 1),
]


@pytest.mark.parametrize("B,H,W,C,L2,kh,kw,stride,pad", CONV_CASES)
def test_unroll(B, H, W, C, L2, kh, kw, stride, pad):
    rng = np.random.default_rng(B + 10 * H + 100 * C + kh)
    x = _pm1(rng, (B, H, W, C))
    got = esp.packed_to_numpy(esp.unroll(_packed_dev(x), C, kh, kw, stride, pad))
    low = oracle.unroll_pm1(x, kh, kw, stride, pad, -1)
    # the packed lowered matrix pads every tap to whole words
    want = oracle.pack_bits(low.reshape(low.shape[0], kh * kw, C)).reshape(low.shape[0], -1)
    assert got.shape == want.shape
    assert np.array_equal(got, want)


@pytest.mark.parametrize("B,H,W,C,L2,kh,kw,stride,pad", CONV_CASES)
def test_bconv(B, H, W, C, L2, kh, kw, stride, pad):
    rng = np.random.default_rng(B + 10 * H + 100 * C + kh + 1000 * L2)
    x = _pm1(rng, (B, H, W, C))
    f = _pm1(rng, (L2, kh, kw, C))
    got = esp.bconv(_packed_dev(x), _packed_dev(f), C, stride, pad).cpu().numpy()
    want = oracle.conv_pm1(x, f, stride, pad, -1)
    assert got.shape == want.shape
    assert np.array_equal(got, want)


def test_bconv_workspace_too_small_is_an_error():
    x = torch.zeros((1, 4, 4, 1), dtype=esp.PACKED, device=DEV)
    f = torch.zeros((2, 3, 3, 1), dtype=esp.PACKED, device=DEV)
    ws = torch.empty(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(esp.EspressoError) as e:
        esp.bconv(x, f, 64, 1, 1, workspace=ws)
    assert e.value.status == -4


def test_config2_conv_bn_sign_pack_chain():
    x, f, bnp = synth.config2()
    xp = esp.pack_f32(_f32(x))
    fp = esp.pack_f32(_f32(f))
    assert np.array_equal(esp.packed_to_numpy(xp), oracle.pack_bits(x))
    pre = esp.bconv(xp, fp, 128, 1, 1)
    want_pre = oracle.conv_pm1(x, f, 1, 1, -1)
    assert np.array_equal(pre.cpu().numpy(), want_pre)
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    bits = esp.bn_sign_pack(pre, torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV))
    want_bits = oracle.pack_bits(oracle.bn_sign(want_pre, bnp, synth.BN_EPS))
    assert bits.shape == (32, 32, 32, 2)
    assert np.array_equal(esp.packed_to_numpy(bits), want_bits)


# ------------------------------------------------------------------------------ bn_sign_pack
# C a multiple of 64 takes the flat-word kernel: with the per-channel state fetched once (words per
# row dividing 16: 64, 128, 1024), carried along (1280 = 20 words: a task wraps inside a row; 1536),
# or the column-per-wave kernel (192 = 3 words; ragged C); row counts leave a partial last task
@pytest.mark.parametrize("rows,C,K", [(1, 64, 64), (5, 70, 300), (64, 4096, 4096), (1000, 128, 1152),
                                      (17, 1024, 8192), (3, 10, 1024), (37, 1280, 2000), (11, 1536, 500),
                                      (50, 192, 900), (3, 128, 128), (7, 256, 700)])
def test_bn_sign_pack(rows, C, K):
    rng = np.random.default_rng(rows + C)
    bnp = synth.bn_params(rng, C)
    # values of the right parity and range for a +-1 dot product of length K, dense near 0
    x = (rng.integers(-min(K, 60), min(K, 60) + 1, size=(rows, C)) * 2 + (K % 2)).astype(np.int32)
    x[0, :] = K
    x[-1, :] = -K
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    got = esp.bn_sign_pack(torch.from_numpy(x).to(DEV), torch.from_numpy(thr).to(DEV),
                           esp.to_packed_tensor(flip, DEV))
    want = oracle.pack_bits(oracle.bn_sign(x, bnp, synth.BN_EPS))
    assert np.array_equal(esp.packed_to_numpy(got), want)


# ------------------------------------------------------------------------------ fused epilogues
# M <= 8 takes the small-M kernel (64 rows of B per block): every row-split it has (K from one
# chunk per row to several chunks per lane), odd word counts, ragged N, and M = 1, 2, 4, 8 and between
SMALL_M_BITS = [(1, 4096, 4096), (2, 100, 70), (3, 1024, 1024), (4, 130, 192), (5, 7, 1000), (8, 1024, 8192),
                (8, 65, 1), (7, 33, 200), (1, 1000, 65472), (2, 129, 20000), (6, 64, 640), (1, 10, 320),
                (1, 16400, 256), (3, 16384, 64), (2, 300, 128)]


@pytest.mark.parametrize("engine", [0, 1])
@pytest.mark.parametrize("M,N,K", SMALL_M_BITS + [(1, 64, 64), (9, 10, 4096), (64, 4096, 1024), (130, 70, 200), (257, 513, 1152),
                                   (1000, 128, 1152), (5, 1024, 8192), (1024, 1024, 1024),
                                   (64, 70, (1 << 20) + 64)])    # K >= 2^20: integer threshold compare on the matrix cores
def test_bgemm_bn_sign_pack(M, N, K, engine):
    rng = np.random.default_rng(M * 31 + N * 17 + K)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    bnp = synth.bn_params(rng, N)
    # make thresholds fall inside the populated range of dot products (|dot| ~ sqrt(K))
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(K)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    got = esp.bgemm_bn_sign_pack(_packed_dev(a), _packed_dev(b), K, torch.from_numpy(thr).to(DEV),
                                 esp.to_packed_tensor(flip, DEV), engine=engine)
    want = oracle.pack_bits(oracle.bn_sign(oracle.dense_pm1(a, b), bnp, synth.BN_EPS))
    assert got.shape == want.shape
    assert np.array_equal(esp.packed_to_numpy(got), want)


# products with few rows take the kernel that splits K over the waves of a block (lane = row,
# 8 columns = one output byte per block): K from one 16-byte chunk to more chunks than waves,
# M around the 64-row groups, N around the byte and word boundaries
@pytest.mark.parametrize("M,N,K", [(9, 8, 128), (63, 9, 256), (64, 64, 4608), (65, 71, 2304), (200, 130, 1152),
                                   (256, 256, 2304), (1000, 100, 384), (33, 500, 8192 + 128), (12, 1024, 8192),
                                   # more blocks than compute units: 8 waves per block instead of 16
                                   (200, 1000, 8192 + 128), (64, 4096, 4096), (100, 2100, 640)])
def test_bgemm_bn_sign_pack_few_rows(M, N, K):
    rng = np.random.default_rng(M * 3 + N * 5 + K)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    bnp = synth.bn_params(rng, N)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(K)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    got = esp.bgemm_bn_sign_pack(_packed_dev(a), _packed_dev(b), K, torch.from_numpy(thr).to(DEV),
                                 esp.to_packed_tensor(flip, DEV))
    want = oracle.pack_bits(oracle.bn_sign(oracle.dense_pm1(a, b), bnp, synth.BN_EPS))
    assert np.array_equal(esp.packed_to_numpy(got), want)


def _random_dense_shape(rng):
    """(M, N, K) with every dimension drawn from one of three ranges: a handful, a few hundred, thousands."""
    def pick(hi):
        r = rng.random()
        if r < 0.25:
            return int(rng.integers(1, 17))
        if r < 0.5:
            return int(rng.integers(17, 300))
        return int(rng.integers(300, hi))
    while True:
        M, N, K = pick(3000), pick(3000), pick(9000)
        if M * N * K <= 2.5e10:
            return M, N, K


# seeded random shapes across the kernels' regimes (matrix-vector, few rows, small and large tiles,
# ragged K and N), every engine: int32 dots and thresholded bits against the oracle
@pytest.mark.parametrize("seed", range(16))
def test_bgemm_random_shapes_all_engines(seed):
    rng = np.random.default_rng(4100 + seed)
    M, N, K = _random_dense_shape(rng)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    want = oracle.dense_pm1(a, b)
    ap, bp = _packed_dev(a), _packed_dev(b)
    assert np.array_equal(esp.bgemm(ap, bp, K).cpu().numpy(), want), (M, N, K)
    assert np.array_equal(esp.bgemm_mfma(ap, bp, K).cpu().numpy(), want), (M, N, K)
    bnp = synth.bn_params(rng, N)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(K)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    thr_d, flip_d = torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV)
    want_bits = oracle.pack_bits(oracle.bn_sign(want, bnp, synth.BN_EPS))
    for engine in (esp.ENGINE_XOR_POPCOUNT, esp.ENGINE_MFMA, esp.ENGINE_AUTO):
        got = esp.bgemm_bn_sign_pack(ap, bp, K, thr_d, flip_d, engine=engine)
        assert np.array_equal(esp.packed_to_numpy(got), want_bits), (M, N, K, engine)


@pytest.mark.parametrize("engine,M,N,K", [(0, 2900, 2950, 640), (1, 2900, 2950, 640),
                                          (0, 2100, 1990, 640), (0, 32768 + 70, 100, 1152)])   # 128x64 tiles
def test_bgemm_bn_sign_pack_large_tiles(engine, M, N, K):
    rng = np.random.default_rng(77)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    bnp = synth.bn_params(rng, N)
    bnp = (bnp[0], bnp[1], (bnp[2] * 25).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    got = esp.bgemm_bn_sign_pack(_packed_dev(a), _packed_dev(b), K, torch.from_numpy(thr).to(DEV),
                                 esp.to_packed_tensor(flip, DEV), engine=engine)
    want = oracle.pack_bits(oracle.bn_sign(oracle.dense_pm1(a, b), bnp, synth.BN_EPS))
    assert np.array_equal(esp.packed_to_numpy(got), want)


FUSED_CONV_CASES = CONV_CASES + [
    (2, 32, 32, 128, 128, 3, 3, 1, 1),     # implicit gather, 32x64 tiles
    (8, 32, 32, 128, 128, 3, 3, 1, 1),     # implicit gather, 64x64 tiles
    (40, 32, 32, 128, 256, 3, 3, 1, 1),    # implicit gather, 128x128 tiles, several K stages
    (33, 32, 32, 128, 100, 3, 3, 1, 1),    # implicit gather, 128x64 tiles, partial word
    (3, 7, 9, 256, 100, 3, 3, 2, 1),
    (2, 5, 5, 384, 64, 3, 3, 1, 1),
]


@pytest.mark.parametrize("engine", [0, 1])
@pytest.mark.parametrize("B,H,W,C,L2,kh,kw,stride,pad", FUSED_CONV_CASES)
def test_bconv_bn_sign_pack(B, H, W, C, L2, kh, kw, stride, pad, engine):
    rng = np.random.default_rng(B + 10 * H + 100 * C + kh + 1000 * L2 + 5)
    x = _pm1(rng, (B, H, W, C))
    f = _pm1(rng, (L2, kh, kw, C))
    bnp = synth.bn_params(rng, L2)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(kh * kw * C)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    xp, fp = _packed_dev(x), _packed_dev(f)
    got = esp.bconv_bn_sign_pack(xp, fp, C, torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV),
                                 stride, pad, engine=engine)
    pre = oracle.conv_pm1(x, f, stride, pad, -1)
    want = oracle.pack_bits(oracle.bn_sign(pre, bnp, synth.BN_EPS))
    assert got.shape == want.shape
    assert np.array_equal(esp.packed_to_numpy(got), want)
    # the int32 route through the same loader
    assert np.array_equal(esp.bconv(xp, fp, C, stride, pad, engine=engine).cpu().numpy(), pre)


# convolution + threshold + sign + 2x2 OR max-pool in one kernel.  Cases: all three tile shapes
# of the XOR-popcount kernel (32, 64 and 128 rows), the pooled widths of the Sec. 6.3 network
# (32, 16, 8), a ragged last tile (M not a multiple of the tile), L2 with a partial last word,
# a 2-pixel-wide output, stride 2, and the largest fusable width (64).
POOL_CONV_CASES = [
    (1, 32, 32, 128, 128, 3, 3, 1, 1),     # batch 1, W2 = 32: forced onto 64-row tiles
    (1, 16, 16, 256, 256, 3, 3, 1, 1),     # W2 = 16: 32-row tiles
    (3, 8, 8, 512, 512, 3, 3, 1, 1),       # W2 = 8
    (40, 32, 32, 128, 256, 3, 3, 1, 1),    # 128-row tiles, several K stages
    (32, 32, 32, 128, 128, 3, 3, 1, 1),    # 128x64 tiles (one word wide)
    (5, 16, 16, 128, 100, 3, 3, 1, 1),     # partial last word, ragged tile count
    (3, 4, 2, 128, 70, 3, 3, 1, 1),        # W2 = 2, H2 = 4
    (2, 16, 8, 128, 64, 3, 3, 2, 1),       # stride 2: H2 = 8, W2 = 4
    (1, 6, 64, 128, 64, 3, 3, 1, 1),       # W2 = 64: 128-row tiles although the product is small
    (7, 2, 2, 256, 192, 1, 1, 1, 0),       # 1x1 filter, one pooled pixel per image
    (2, 8, 32, 128, 72, 3, 3, 1, 1),       # few rows, W2 = 32: pool partners in the other half-wave
    (1, 10, 4, 384, 200, 3, 3, 1, 1),      # few rows, H2 = 10: last 64-row group half empty
    (1, 4, 64, 128, 16, 3, 3, 1, 1),       # few rows but W2 = 64: tiled kernel
]


@pytest.mark.parametrize("engine", [0, 1, 2])
@pytest.mark.parametrize("B,H,W,C,L2,kh,kw,stride,pad", POOL_CONV_CASES)
def test_bconv_bn_sign_pack_pool2(B, H, W, C, L2, kh, kw, stride, pad, engine):
    rng = np.random.default_rng(B + 10 * H + 100 * C + kh + 1000 * L2 + 11)
    x = _pm1(rng, (B, H, W, C))
    f = _pm1(rng, (L2, kh, kw, C))
    bnp = synth.bn_params(rng, L2)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(kh * kw * C)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    assert esp.bconv_pool2_fusable(H, W, C, kh, kw, stride, pad)
    xp, fp = _packed_dev(x), _packed_dev(f)
    got = esp.bconv_bn_sign_pack_pool2(xp, fp, C, torch.from_numpy(thr).to(DEV),
                                       esp.to_packed_tensor(flip, DEV), stride, pad, engine=engine)
    act = oracle.bn_sign(oracle.conv_pm1(x, f, stride, pad, -1), bnp, synth.BN_EPS)
    want = oracle.pack_bits(oracle.maxpool_pm1(act, 2, 2))
    assert got.shape == want.shape
    assert np.array_equal(esp.packed_to_numpy(got), want)


# Stride-1 layers with at least 512 tiles of 128 pixels x 64 filters take the kernel that keeps the
# filters in LDS and streams the input as patches (whole image rows per tile).  Cases: tiles inside
# one image and tiles of two whole images with an odd batch (a half-empty last tile); 128, 256 and
# 512 channels; a partial last word of filters; output widths 8, 16, 32 and 128; 1x1, 3x3, 5x5 and
# 1x3 filters; blocks that walk 1, 2, 3 and 8 row tiles.  int32, thresholded and pooled outputs.
PATCH_CONV_CASES = [
    # B, H, W, C, L2, kh, kw, pad
    (40, 32, 32, 128, 256, 3, 3, 1),
    (33, 32, 32, 128, 100, 3, 3, 1),
    (129, 8, 8, 128, 512, 3, 3, 1),
    (64, 16, 16, 256, 256, 3, 3, 1),
    (128, 2, 128, 128, 128, 3, 3, 1),
    (256, 16, 16, 128, 64, 1, 1, 0),
    (64, 32, 32, 128, 64, 5, 5, 2),
    (150, 14, 16, 128, 128, 1, 3, 1),
    (2048, 16, 16, 512, 64, 3, 3, 1),
    # 128 filters per block (8 x 8 counters per lane): one, two and three filter tiles, a ragged
    # last row tile of two-image tiles, 128 and 256 channels
    (72, 32, 32, 128, 128, 3, 3, 1),
    (261, 8, 8, 256, 512, 3, 3, 1),
    (130, 16, 16, 128, 384, 3, 3, 1),
    # 512 channels, 128 filters per block: blocks of two halves that walk pairs of row tiles; an odd
    # number of row tiles (the last pair's second half has nothing to store), two-image tiles
    (129, 8, 8, 512, 1024, 3, 3, 1),
    (66, 16, 16, 512, 512, 3, 3, 1),
]


@pytest.mark.parametrize("B,H,W,C,L2,kh,kw,pad", PATCH_CONV_CASES)
def test_bconv_whole_row_tiles(B, H, W, C, L2, kh, kw, pad):
    rng = np.random.default_rng(B + 10 * H + 100 * C + kh + 1000 * L2 + 17)
    x = _pm1(rng, (B, H, W, C))
    f = _pm1(rng, (L2, kh, kw, C))
    bnp = synth.bn_params(rng, L2)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(kh * kw * C)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    thr_d, flip_d = torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV)
    xp, fp = _packed_dev(x), _packed_dev(f)
    pre = oracle.conv_pm1(x, f, 1, pad, -1)
    assert np.array_equal(esp.bconv(xp, fp, C, 1, pad).cpu().numpy(), pre)
    act = oracle.bn_sign(pre, bnp, synth.BN_EPS)
    del pre
    got = esp.bconv_bn_sign_pack(xp, fp, C, thr_d, flip_d, 1, pad)
    assert np.array_equal(esp.packed_to_numpy(got), oracle.pack_bits(act))
    if esp.bconv_pool2_fusable(H, W, C, kh, kw, 1, pad):
        got = esp.bconv_bn_sign_pack_pool2(xp, fp, C, thr_d, flip_d, 1, pad)
        assert np.array_equal(esp.packed_to_numpy(got), oracle.pack_bits(oracle.maxpool_pm1(act, 2, 2)))


def _random_whole_row_shape(rng):
    """A stride-1 layer that qualifies for the whole-row-tile kernels: 128 / 256 / 512 channels, output
    width a power of two, output pixels per image a multiple or a divisor of 128, at least 512 tiles."""
    while True:
        C = int(rng.choice([128, 256, 512]))
        W = int(rng.choice([8, 16, 32, 64]))
        kh, kw = int(rng.choice([1, 3, 3, 3, 5])), int(rng.choice([1, 3, 3, 3, 5]))
        pad = int(rng.choice([0, 1, 2]))
        W2 = W + 2 * pad - kw + 1
        if W2 < 8 or (W2 & (W2 - 1)):
            continue
        H2 = int(rng.choice([h for h in range(1, 65) if (h * W2) % 128 == 0 or 128 % (h * W2) == 0]))
        H = H2 - 2 * pad + kh - 1
        if H < 1:
            continue
        L2 = int(rng.choice([64, 100, 128, 200, 256, 384, 512]))
        tiles_per_image = H2 * W2 / 128.0
        B = int(np.ceil(512 / tiles_per_image / ((L2 + 63) // 64))) + int(rng.integers(0, 3))
        if B * H2 * W2 * L2 * kh * kw * C <= 3e10 and B * H * W * C <= 2e8:
            return B, H, W, C, L2, kh, kw, pad


# seeded random shapes on top of the hand-picked ones above: filter heights and widths that differ,
# no padding or more than the filter needs, tiles of several images, ragged last tiles, filter
# counts that are no multiple of 64
@pytest.mark.parametrize("seed", range(12))
def test_bconv_whole_row_tiles_random_shapes(seed):
    rng = np.random.default_rng(9000 + seed)
    B, H, W, C, L2, kh, kw, pad = _random_whole_row_shape(rng)
    x = _pm1(rng, (B, H, W, C))
    f = _pm1(rng, (L2, kh, kw, C))
    bnp = synth.bn_params(rng, L2)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(kh * kw * C)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    thr_d, flip_d = torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV)
    xp, fp = _packed_dev(x), _packed_dev(f)
    pre = oracle.conv_pm1(x, f, 1, pad, -1)
    assert np.array_equal(esp.bconv(xp, fp, C, 1, pad).cpu().numpy(), pre), (B, H, W, C, L2, kh, kw, pad)
    act = oracle.bn_sign(pre, bnp, synth.BN_EPS)
    del pre
    got = esp.bconv_bn_sign_pack(xp, fp, C, thr_d, flip_d, 1, pad)
    assert np.array_equal(esp.packed_to_numpy(got), oracle.pack_bits(act)), (B, H, W, C, L2, kh, kw, pad)
    if esp.bconv_pool2_fusable(H, W, C, kh, kw, 1, pad):
        got = esp.bconv_bn_sign_pack_pool2(xp, fp, C, thr_d, flip_d, 1, pad)
        assert np.array_equal(esp.packed_to_numpy(got), oracle.pack_bits(oracle.maxpool_pm1(act, 2, 2)))


def test_bconv_pool2_rejects_shapes_it_cannot_fuse():
    assert not esp.bconv_pool2_fusable(32, 32, 64, 3, 3, 1, 1)     # lowered-matrix path
    assert not esp.bconv_pool2_fusable(7, 8, 128, 3, 3, 1, 1)      # odd output height
    assert not esp.bconv_pool2_fusable(8, 12, 128, 3, 3, 1, 1)     # width not a power of two
    assert not esp.bconv_pool2_fusable(8, 128, 128, 3, 3, 1, 1)    # a row pair exceeds the tile
    rng = np.random.default_rng(3)
    x = _packed_dev(_pm1(rng, (1, 8, 12, 128)))
    f = _packed_dev(_pm1(rng, (64, 3, 3, 128)))
    thr = torch.zeros(64, dtype=torch.int32, device=DEV)
    flip = torch.zeros(1, dtype=esp.PACKED, device=DEV)
    with pytest.raises(esp.EspressoError):
        esp.bconv_bn_sign_pack_pool2(x, f, 128, thr, flip, 1, 1)


# ------------------------------------------------------------------------------ zero-padding correction
PADCORR_CASES = [(2, 5, 6, 128, 7, 3, 3, 1, 1), (2, 7, 5, 192, 5, 3, 3, 2, 1), (1, 6, 6, 100, 9, 3, 3, 1, 1),
                 (2, 9, 7, 256, 64, 5, 3, 2, 2), (3, 32, 32, 128, 128, 3, 3, 1, 1), (2, 8, 8, 64, 12, 3, 3, 1, 0),
                 (1, 3, 3, 64, 4, 3, 3, 1, 2), (2, 6, 7, 64, 6, 2, 2, 2, 1)]


@pytest.mark.parametrize("B,H,W,C,L2,kh,kw,stride,pad", PADCORR_CASES)
def test_pad_correction(B, H, W, C, L2, kh, kw, stride, pad):
    # (-1)-padded convolution + correction matrix == zero-padded convolution (Sec. 5.2)
    rng = np.random.default_rng(B + 10 * H + 100 * C + kh + 7)
    x = _pm1(rng, (B, H, W, C))
    f = _pm1(rng, (L2, kh, kw, C))
    xp, fp = _packed_dev(x), _packed_dev(f)
    corr = esp.pad_correction(fp, C, H, W, stride, pad)
    want_corr = oracle.conv_pm1(np.zeros((1, H, W, C), dtype=np.int8), f, stride, pad, +1)[0]
    assert np.array_equal(corr.cpu().numpy(), want_corr)
    out = esp.bconv(xp, fp, C, stride, pad)
    esp.add_pad_correction(out, corr, H, W, kh, kw, stride, pad)
    assert np.array_equal(out.cpu().numpy(), oracle.conv_pm1(x, f, stride, pad, 0))


# ------------------------------------------------------------------------------ bit-plane first layer
@pytest.mark.parametrize("M,N,K", [(1, 10, 64), (3, 70, 100), (64, 4096, 784), (9, 130, 1000), (1, 4096, 784)])
def test_bitplane_dense(M, N, K):
    rng = np.random.default_rng(M + N + K)
    x = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    x[0, : min(K, 4)] = [0, 255, 1, 128][: min(K, 4)]
    w = _pm1(rng, (N, K))
    wp = _packed_dev(w)
    planes = esp.bitplane_pack_u8(torch.from_numpy(x).to(DEV))
    assert planes.shape == (M, 8, (K + 63) // 64)
    want_planes = np.stack([oracle.pack_bits((((x >> i) & 1).astype(np.int8) * 2 - 1)) for i in range(8)], axis=1)
    assert np.array_equal(esp.packed_to_numpy(planes), want_planes)
    wsum = esp.row_sums(wp, K)
    assert np.array_equal(wsum.cpu().numpy(), w.astype(np.int64).sum(axis=1))
    d = esp.bgemm(planes.reshape(M * 8, -1), wp, K).reshape(M, 8, N)
    y = esp.bitplane_combine(d, wsum)
    assert np.array_equal(y.cpu().numpy(), oracle.dense_u8(x, w))


# the same layer as ONE call on the matrix cores (planes combined in the product's epilogue): y and
# the thresholded sign bits against the oracle's exact integer layer; row counts and widths that leave
# partial tiles, K with an odd number of words (8-byte loads), both block shapes
@pytest.mark.parametrize("M,N,K", [(1, 10, 64), (3, 70, 200), (64, 4096, 784), (33, 130, 1000), (300, 257, 832),
                                   (1024, 4096, 784), (5, 64, 4096)])
def test_bitplane_dense_fused(M, N, K):
    rng = np.random.default_rng(M + 3 * N + 5 * K)
    x = rng.integers(0, 256, size=(M, K), dtype=np.uint8)
    x[0, : min(K, 4)] = [0, 255, 1, 128][: min(K, 4)]
    w = _pm1(rng, (N, K))
    wp = _packed_dev(w)
    planes = esp.bitplane_pack_u8(torch.from_numpy(x).to(DEV))
    wsum = esp.row_sums(wp, K)
    want = oracle.dense_u8(x, w)
    bnp = synth.bn_params(rng, N)
    bnp = (bnp[0], bnp[1], (bnp[2] * 40 * np.sqrt(K)).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    thr_d, flip_d = torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV)
    want_bits = oracle.pack_bits(oracle.bn_sign(want, bnp, synth.BN_EPS))
    bits, y = esp.bitplane_dense(planes, wp, wsum, K, thr=thr_d, flip=flip_d, want_y=True)
    assert np.array_equal(y.cpu().numpy(), want)
    assert np.array_equal(esp.packed_to_numpy(bits), want_bits)
    bits_only, none = esp.bitplane_dense(planes, wp, wsum, K, thr=thr_d, flip=flip_d)
    assert none is None and torch.equal(bits_only, bits)
    none, y_only = esp.bitplane_dense(planes, wp, wsum, K, want_y=True)
    assert none is None and torch.equal(y_only, y)


@pytest.mark.parametrize("B,H,W,C,L2", [(2, 32, 32, 3, 128), (3, 6, 5, 3, 20), (1, 8, 8, 70, 9)])
def test_bitplane_conv(B, H, W, C, L2):
    rng = np.random.default_rng(B + H + C + L2)
    x = rng.integers(0, 256, size=(B, H, W, C), dtype=np.uint8)
    f = _pm1(rng, (L2, 3, 3, C))
    fp = _packed_dev(f)
    planes = esp.bitplane_pack_u8(torch.from_numpy(x).to(DEV))          # [B][8][H][W][Cw]
    assert planes.shape == (B, 8, H, W, (C + 63) // 64)
    wsum = esp.row_sums(fp, 9 * C)      # every tap is padded to whole words; tail bits are 0
    assert np.array_equal(wsum.cpu().numpy(), f.reshape(L2, -1).astype(np.int64).sum(axis=1))
    d = esp.bconv(planes.reshape(B * 8, H, W, -1), fp, C, 1, 1).reshape(B, 8, H, W, L2)
    y = esp.bitplane_combine(d, wsum)
    assert np.array_equal(y.cpu().numpy(), oracle.conv_u8(x, f, 1, 1))


# ------------------------------------------------------------------------------ bmaxpool
@pytest.mark.parametrize("B,H,W,C,win,stride", [(1, 2, 2, 64, 2, 2), (2, 8, 8, 128, 2, 2), (3, 7, 9, 192, 2, 2),
                                                (2, 6, 6, 100, 3, 1), (4, 32, 32, 128, 2, 2),
                                                (2, 8, 8, 512, 2, 2), (1, 9, 9, 64, 3, 3)])
def test_bmaxpool(B, H, W, C, win, stride):
    rng = np.random.default_rng(B * 31 + H + C)
    # mostly -1 so that all-(-1) windows occur
    x = np.where(rng.random((B, H, W, C)) < 0.25, 1, -1).astype(np.int8)
    got = esp.packed_to_numpy(esp.bmaxpool(_packed_dev(x), C, win, stride))
    want = oracle.pack_bits(oracle.maxpool_pm1(x, win, stride))
    assert got.shape == want.shape
    assert np.array_equal(got, want)


# ------------------------------------------------------------------------------ float first layer
def _assert_close_1e4(got, ref):
    err = np.abs(got.astype(np.float64) - ref)
    tol = 1e-4 * np.maximum(1.0, np.abs(ref))
    assert np.all(err <= tol), float((err / tol).max())


@pytest.mark.parametrize("M,N,K", [(1, 4096, 784), (3, 100, 50), (64, 4096, 784), (70, 130, 97), (4, 10, 784),
                                   (1024, 4096, 784), (300, 1000, 130), (65, 33, 36), (5, 64, 31), (2000, 700, 100),
                                   # 256 rows and more: the three-term bf16 kernel; K not a multiple of 4 or of
                                   # its 64-wide slabs, ragged M and N, 64- and 128-row tiles
                                   (256, 128, 64), (257, 130, 97), (300, 70, 131), (4100, 2050, 70), (8200, 8100, 40)])
def test_dense_f32(M, N, K):
    rng = np.random.default_rng(M + N + K)
    x = rng.random((M, K), dtype=np.float32)
    w = _pm1(rng, (N, K))
    got = esp.dense_f32(_f32(x), _f32(w)).cpu().numpy()
    _assert_close_1e4(got, oracle.dense_f64(x, w))


# 3x3x3 stride-1 shapes take the matrix-core kernel: one to four 32-channel blocks, several
# channel groups, strips of 32 pixels with a ragged last strip, pad 0, 1 and 2
CONV3_CASES = [(2, 40, 70, 3, 200, 3, 1, 1), (1, 5, 5, 3, 32, 3, 1, 0), (2, 6, 6, 3, 48, 3, 1, 2),
               (3, 4, 33, 3, 129, 3, 1, 1), (5, 32, 32, 3, 128, 3, 1, 1), (1, 3, 3, 3, 7, 3, 1, 0)]


@pytest.mark.parametrize("B,H,W,C,L2,k,stride,pad", [(1, 32, 32, 3, 128, 3, 1, 1), (3, 9, 7, 3, 20, 3, 2, 1),
                                                     (2, 8, 8, 5, 300, 3, 1, 0), (2, 6, 6, 16, 2000, 3, 1, 1)]
                         + CONV3_CASES)
def test_conv_f32(B, H, W, C, L2, k, stride, pad):
    rng = np.random.default_rng(B + H + L2)
    x = rng.random((B, H, W, C), dtype=np.float32)
    f = _pm1(rng, (L2, k, k, C))
    got = esp.conv_f32(_f32(x), _f32(f), stride, pad).cpu().numpy()
    _assert_close_1e4(got, oracle.conv_f64(x, f, stride, pad))


@pytest.mark.parametrize("M,N,K", [(1, 4096, 784), (2, 100, 50), (3, 64, 31), (4, 130, 784), (1, 65, 4),
                                   (4, 1000, 1001), (5, 4096, 784), (70, 130, 97), (2, 16390, 64),
                                   (64, 4096, 784), (1024, 4096, 784), (300, 70, 130), (65, 33, 36),
                                   (256, 128, 64), (257, 130, 97), (8200, 4000, 40), (300, 200, 131)])
def test_dense_f32_bn_sign_pack(M, N, K):
    # M <= 4: the streaming kernel (16 or 64 neurons per block); beyond: the matrix-core kernel
    rng = np.random.default_rng(M + 10 * N + 100 * K)
    x = rng.random((M, K), dtype=np.float32)
    w = _pm1(rng, (N, K))
    bnp = synth.bn_params(rng, N)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(K) + 0.5 * w.sum(axis=1)).astype(np.float32), bnp[3])
    thr, sgn = esp.bn_fold_f32(*bnp, synth.BN_EPS)
    xd, wd, td, sd = _f32(x), _f32(w), _f32(thr), _f32(sgn)
    pre = torch.empty((M, N), dtype=torch.float32, device=DEV)
    bits = esp.dense_f32_bn_sign_pack(xd, wd, td, sd, pre=pre)
    _assert_close_1e4(pre.cpu().numpy(), oracle.dense_f64(x, w))
    # bits equal the oracle's batch-norm + sign of those same fp32 pre-activations
    want = oracle.pack_bits(oracle.bn_sign(pre.cpu().numpy().astype(np.float64), bnp, synth.BN_EPS))
    assert np.array_equal(esp.packed_to_numpy(bits), want)
    assert torch.equal(esp.dense_f32_bn_sign_pack(xd, wd, td, sd), bits)      # without `pre`


@pytest.mark.parametrize("M,N,K", [(1, 4096, 784), (2, 100, 50), (3, 64, 31), (4, 130, 784), (1, 65, 4),
                                   (4, 1000, 1001), (5, 4096, 784), (70, 130, 97), (2, 16390, 64),
                                   (64, 4096, 784), (1024, 4096, 784), (300, 70, 130), (65, 33, 36),
                                   (257, 130, 97), (300, 200, 131), (1, 10, 1), (3, 70, 129)])
def test_dense_f32_bw_bn_sign_pack(M, N, K):
    # the same layer with its +-1 weights bit-packed
    rng = np.random.default_rng(7 + M + 10 * N + 100 * K)
    x = (rng.random((M, K), dtype=np.float32) - 0.25).astype(np.float32)
    w = _pm1(rng, (N, K))
    bnp = synth.bn_params(rng, N)
    bnp = (bnp[0], bnp[1], (bnp[2] * np.sqrt(K) + 0.25 * w.sum(axis=1)).astype(np.float32), bnp[3])
    thr, sgn = esp.bn_fold_f32(*bnp, synth.BN_EPS)
    xd, wb, td, sd = _f32(x), _packed_dev(w), _f32(thr), _f32(sgn)
    pre = torch.empty((M, N), dtype=torch.float32, device=DEV)
    bits = esp.dense_f32_bw_bn_sign_pack(xd, wb, td, sd, pre=pre)
    _assert_close_1e4(pre.cpu().numpy(), oracle.dense_f64(x, w))
    want = oracle.pack_bits(oracle.bn_sign(pre.cpu().numpy().astype(np.float64), bnp, synth.BN_EPS))
    assert np.array_equal(esp.packed_to_numpy(bits), want)
    assert torch.equal(esp.dense_f32_bw_bn_sign_pack(xd, wb, td, sd), bits)      # without `pre`


@pytest.mark.parametrize("M", [3, 70, 600])
def test_dense_f32_bn_sign_pack_wide_dynamic_range(M):
    # signed inputs spread over six decades, exact zeros, values with all 24 significand bits set:
    # the three-term bf16 kernel (M > 4) must stay within the fp32 tolerance like the streaming one
    N, K = 200, 777
    rng = np.random.default_rng(M)
    x = (rng.standard_normal((M, K)) * 10.0 ** rng.uniform(-3, 3, size=(M, K))).astype(np.float32)
    x[rng.random((M, K)) < 0.05] = 0.0
    x[0, :8] = np.float32(1.9999999)       # 0x3fffffff: every significand bit set
    x[0, 8:16] = np.float32(-16777215.0)   # 2^24 - 1
    w = _pm1(rng, (N, K))
    pre = torch.empty((M, N), dtype=torch.float32, device=DEV)
    thr, sgn = np.zeros(N, np.float32), np.ones(N, np.float32)
    esp.dense_f32_bn_sign_pack(_f32(x), _f32(w), _f32(thr), _f32(sgn), pre=pre)
    ref = oracle.dense_f64(x, w)
    got = pre.cpu().numpy().astype(np.float64)
    # error of a sum of K exact products accumulated in fp32, relative to the sum of magnitudes
    scale = np.abs(x.astype(np.float64)).sum(axis=1, keepdims=True)
    assert np.all(np.abs(got - ref) <= 1e-6 * scale + 1e-30)


def test_bn_sign_pack_f32_bit_exact_on_given_preactivations():
    # Batch-norm + sign is folded on the host to a float threshold per channel that is exact
    # for every float input, so on the SAME float32 pre-activations the bits equal the
    # oracle's double-precision batch-norm + sign, ties and near-ties included.
    rng = np.random.default_rng(3)
    rows, C = 300, 200
    bnp = synth.bn_params(rng, C)
    x = (rng.standard_normal((rows, C)) * 20).astype(np.float32)
    g, b, m, v = bnp
    # plant exact zeros of y: gamma * (x - mean) / s + beta == 0 needs beta = 0, x = mean
    b[:5] = 0.0
    x[:, :5] = m[:5]
    thr, sgn = esp.bn_fold_f32(g, b, m, v, synth.BN_EPS)
    # plant values at and next to every threshold (both sides)
    t = np.where(np.isfinite(thr), sgn * thr, 0.0).astype(np.float32)
    x[5, :] = t
    x[6, :] = np.nextafter(t, np.float32(np.inf))
    x[7, :] = np.nextafter(t, np.float32(-np.inf))
    x[8, :] = 0.0
    x[9, :] = -0.0
    got = esp.bn_sign_pack_f32(_f32(x), _f32(thr), _f32(sgn))
    want = oracle.pack_bits(oracle.bn_sign(x.astype(np.float64), (g, b, m, v), synth.BN_EPS))
    assert np.array_equal(esp.packed_to_numpy(got), want)


def test_conv_f32_bn_sign_pack_fused_equals_two_step():
    rng = np.random.default_rng(4)
    for (B, H, W, C, L2, k, stride, pad) in [(3, 32, 32, 3, 128, 3, 1, 1), (2, 9, 11, 3, 70, 3, 1, 1),
                                             (2, 8, 8, 5, 40, 3, 1, 0), (1, 7, 7, 3, 64, 3, 2, 1)] + CONV3_CASES:
        x = rng.random((B, H, W, C), dtype=np.float32)
        f = _pm1(rng, (L2, k, k, C))
        bnp = synth.bn_params(rng, L2)
        thr, sgn = esp.bn_fold_f32(*bnp, synth.BN_EPS)
        xd, fd, td, sd = _f32(x), _f32(f), _f32(thr), _f32(sgn)
        pre = esp.conv_f32(xd, fd, stride, pad)
        two = esp.bn_sign_pack_f32(pre, td, sd)
        pre2 = torch.empty_like(pre)
        fused = esp.conv_f32_bn_sign_pack(xd, fd, td, sd, stride, pad, pre=pre2)
        assert torch.equal(pre, pre2)
        assert torch.equal(fused, two)
        # bits equal the oracle's batch-norm + sign of those same fp32 pre-activations
        want = oracle.pack_bits(oracle.bn_sign(pre.cpu().numpy().astype(np.float64), bnp, synth.BN_EPS))
        assert np.array_equal(esp.packed_to_numpy(fused), want)
        if (C, k, stride) == (3, 3, 1):
            assert torch.equal(esp.conv_f32_bn_sign_pack(xd, fd, td, sd, stride, pad), two)


def test_conv3x3x3_wide_dynamic_range():
    # the 3x3x3 matrix-core path (three bf16 terms per input) on signed inputs spread over six
    # decades: error of 27 exact products accumulated in fp32
    rng = np.random.default_rng(11)
    B, H, W, L2 = 2, 20, 37, 100
    x = (rng.standard_normal((B, H, W, 3)) * 10.0 ** rng.uniform(-3, 3, size=(B, H, W, 3))).astype(np.float32)
    x[0, 0, :4, :] = np.float32(1.9999999)
    f = _pm1(rng, (L2, 3, 3, 3))
    got = esp.conv_f32(_f32(x), _f32(f), 1, 1).cpu().numpy().astype(np.float64)
    ref = oracle.conv_f64(x, f, 1, 1)
    scale = oracle.conv_f64(np.abs(x), np.ones_like(f), 1, 1)      # sum of magnitudes per output
    assert np.all(np.abs(got - ref) <= 1e-6 * scale + 1e-30)


def test_xor_popcount_probe_counts_what_it_claims():
    # the measurement aid must really execute the pairs it reports: every lane's counter sum is
    # iters * sum_ij popcount(a_i ^ b_j) for the lane's seeded register values
    blocks, iters = 3, 5
    sink = torch.zeros(blocks * 256, dtype=torch.int32, device=DEV)
    bop = esp.xor_popcount_probe(sink, blocks, iters)
    assert bop == blocks * 256 * iters * 64 * 64
    seed = np.arange(blocks * 256, dtype=np.uint64)
    mask = np.uint64(0xffffffff)
    a = [(seed * np.uint64(2654435761) + np.uint64(0x9e3779b9 * (i + 1))) & mask for i in range(8)]
    b = [(seed * np.uint64(40503) + np.uint64(0x85ebca6b * (j + 1))) & mask for j in range(8)]
    want = np.zeros(blocks * 256, dtype=np.int64)
    for ai in a:
        for bj in b:
            x = ai ^ bj
            want += np.array([bin(int(v)).count("1") for v in x])
    assert np.array_equal(sink.cpu().numpy().astype(np.int64), want * iters)
    # the single-instruction modes: two dependent xors per slot (acc ^= a; acc ^= b: after an odd
    # number of rounds every counter holds a ^ b), two dependent popcount-accumulates per slot
    assert esp.xor_popcount_probe(sink, blocks, iters, esp.PROBE_XOR_ONLY) == blocks * 256 * iters * 64 * 2
    want_x = np.zeros(blocks * 256, dtype=np.uint64)
    for ai in a:
        for bj in b:
            want_x = (want_x + (ai ^ bj)) & mask
    assert np.array_equal(sink.cpu().numpy().view(np.uint32).astype(np.uint64), want_x)
    assert esp.xor_popcount_probe(sink, blocks, iters, esp.PROBE_POPCOUNT_ONLY) == blocks * 256 * iters * 64 * 2
    popc = lambda v: np.array([bin(int(t)).count("1") for t in v])
    want_p = 8 * (sum(popc(ai) for ai in a) + sum(popc(bj) for bj in b))
    assert np.array_equal(sink.cpu().numpy().astype(np.int64), want_p * iters)
