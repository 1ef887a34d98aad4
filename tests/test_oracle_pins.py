"""Pins for the CPU oracle: checks against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each pin is chosen so that a
plausible mistake in the oracle (dropped term, wrong sign or index, transposed
operand, wrong bit order) fails at least one of them.  The paper prints no
worked numeric example; the only numbers it prints that constrain this path are
the memory footprints of Sec. 6.2 / 6.3 (``tests/golden/paper_footprints.txt``).
"""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import nets
from paper_1705_07175_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _pm1(rng, shape):
    return (rng.integers(0, 2, size=shape, dtype=np.int8) * 2 - 1).astype(np.int8)


# ------------------------------------------------------------------ sign / packing
def test_sign_eq1_conventions():
    # Eq. 1: x >= 0 -> +1, otherwise -1; zero and negative zero are >= 0.
    x = np.array([0.0, -0.0, 1e-30, -1e-30, 3.5, -2.0, np.inf, -np.inf, np.nan], dtype=np.float32)
    assert oracle.sign(x).tolist() == [1, 1, 1, -1, 1, -1, 1, -1, -1]
    assert oracle.sign(x.astype(np.float64)).tolist() == [1, 1, 1, -1, 1, -1, 1, -1, -1]


@pytest.mark.parametrize("k", [1, 63, 64, 65, 128, 200])
def test_pack_one_hot_bit_order(k):
    # Sec. 4.1: -1 -> 0, +1 -> 1.  Element i alone at +1 gives word i//64 == 2**(i%64).
    kw = (k + 63) // 64
    for i in range(k):
        s = -np.ones((1, k), dtype=np.int8)
        s[0, i] = 1
        w = oracle.pack_bits(s)
        assert w.shape == (1, kw)
        expect = [0] * kw
        expect[i // 64] = 1 << (i % 64)
        assert [int(v) for v in w[0]] == expect


def test_pack_all_ones_and_tail_zero():
    for k in (1, 64, 70, 127, 128):
        w = oracle.pack_bits(np.ones((2, k), dtype=np.int8))
        total = sum(bin(int(v)).count("1") for v in w[0])
        assert total == k  # tail bits are zero
        assert np.array_equal(w[0], w[1])
    assert int(oracle.pack_bits(-np.ones((1, 64), dtype=np.int8))[0, 0]) == 0


def test_pack_round_trip_and_little_endian_halves():
    rng = np.random.default_rng(1)
    s = _pm1(rng, (5, 3, 200))
    w = oracle.pack_bits(s)
    assert w.shape == (5, 3, 4)
    assert np.array_equal(oracle.unpack_bits(w, 200), s)
    # Independent reading of the same buffer: bit i of a row is bit i%8 of byte i//8.
    bits = np.unpackbits(w.view(np.uint8).reshape(5, 3, -1), axis=-1, bitorder="little")[..., :200]
    assert np.array_equal(bits.astype(np.int8) * 2 - 1, s)


# ------------------------------------------------------------------ binary dense
def _dot_brute(a, b):
    M, K = a.shape
    N = b.shape[0]
    c = [[0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            t = 0
            for k in range(K):
                t += int(a[m][k]) * int(b[n][k])
            c[m][n] = t
    return np.array(c, dtype=np.int32)


@pytest.mark.parametrize("M,N,K", [(1, 1, 64), (2, 3, 128), (3, 2, 192), (3, 5, 7), (4, 1, 65)])
def test_dense_brute_force(M, N, K):
    rng = np.random.default_rng(M * 100 + N * 10 + K)
    a, b = _pm1(rng, (M, K)), _pm1(rng, (N, K))
    assert np.array_equal(oracle.dense_pm1(a, b), _dot_brute(a, b))


def test_dense_hand_example():
    # Worked by hand: a = (+,-,+,+), b0 = (+,+,+,-), b1 = -a.
    a = np.array([[1, -1, 1, 1]], dtype=np.int8)
    b = np.array([[1, 1, 1, -1], [-1, 1, -1, -1]], dtype=np.int8)
    assert oracle.dense_pm1(a, b).tolist() == [[0, -4]]


def test_dense_eq2_identity_mismatch_count():
    # Eq. 2 with the mismatch count: a.b = K - 2 * #(positions where a and b differ).
    rng = np.random.default_rng(2)
    for K in (64, 128, 192, 100):
        a, b = _pm1(rng, (3, K)), _pm1(rng, (4, K))
        c = oracle.dense_pm1(a, b)
        aw, bw = oracle.pack_bits(a), oracle.pack_bits(b)
        for m in range(3):
            for n in range(4):
                d = oracle.mismatches(aw[m], bw[n])
                assert c[m, n] == K - 2 * d
                assert d == int(np.sum(a[m] != b[n]))


def test_dense_closed_forms():
    rng = np.random.default_rng(3)
    K = 320
    a = _pm1(rng, (6, K))
    c = oracle.dense_pm1(a, a)
    assert np.all(np.diag(c) == K)                      # a.a = K
    assert np.array_equal(c, c.T)
    assert np.all(np.diag(oracle.dense_pm1(a, -a)) == -K)   # a.(-a) = -K
    ones = np.ones((2, K), dtype=np.int8)
    assert np.all(oracle.dense_pm1(ones, ones) == K)
    b = _pm1(rng, (9, K))
    c = oracle.dense_pm1(a, b)
    assert np.all((c - K) % 2 == 0) and np.all(np.abs(c) <= K)  # parity and range
    assert np.array_equal(c.T, oracle.dense_pm1(b, a))         # C(A,B)^T = C(B,A)
    # row/column checksums touch every output element
    assert np.array_equal(c.sum(axis=1), a.astype(np.int64) @ b.astype(np.int64).sum(axis=0))
    assert np.array_equal(c.sum(axis=0), b.astype(np.int64) @ a.astype(np.int64).sum(axis=0))


def test_dense_library_third_opinion():
    # float64 matmul of +-1 matrices is exact for K < 2**53.
    rng = np.random.default_rng(4)
    a, b = _pm1(rng, (17, 333)), _pm1(rng, (29, 333))
    ref = (a.astype(np.float64) @ b.astype(np.float64).T).astype(np.int32)
    assert np.array_equal(oracle.dense_pm1(a, b), ref)


def test_dense_threads_do_not_change_result():
    rng = np.random.default_rng(5)
    a, b = _pm1(rng, (33, 130)), _pm1(rng, (21, 130))
    oracle.set_threads(1)
    c1 = oracle.dense_pm1(a, b)
    oracle.set_threads(4)
    try:
        c4 = oracle.dense_pm1(a, b)
    finally:
        oracle.set_threads(1)
    assert np.array_equal(c1, c4)


# ------------------------------------------------------------------ convolution / unrolling
def _conv_brute(x, f, stride, pad, pad_value):
    B, H, W, C = x.shape
    L2, kh, kw, _ = f.shape
    H2 = (H + 2 * pad - kh) // stride + 1
    W2 = (W + 2 * pad - kw) // stride + 1
    xp = np.full((B, H + 2 * pad, W + 2 * pad, C), pad_value, dtype=np.int64)
    xp[:, pad:pad + H, pad:pad + W, :] = x
    out = np.zeros((B, H2, W2, L2), dtype=np.int64)
    for b, m, n, l in itertools.product(range(B), range(H2), range(W2), range(L2)):
        patch = xp[b, m * stride:m * stride + kh, n * stride:n * stride + kw, :]
        out[b, m, n, l] = int(np.sum(patch * f[l].astype(np.int64)))
    return out.astype(np.int32)


@pytest.mark.parametrize("stride,pad,kh,kw", [(1, 1, 3, 3), (1, 0, 3, 3), (2, 1, 3, 3), (1, 2, 5, 3), (2, 0, 2, 2)])
def test_conv_brute_force(stride, pad, kh, kw):
    rng = np.random.default_rng(10 + stride + pad + kh)
    x = _pm1(rng, (2, 5, 6, 4))
    f = _pm1(rng, (3, kh, kw, 4))
    got = oracle.conv_pm1(x, f, stride, pad, -1)
    assert np.array_equal(got, _conv_brute(x, f, stride, pad, -1))


def test_conv_1x1_is_dense():
    rng = np.random.default_rng(11)
    x = _pm1(rng, (2, 4, 5, 64))
    f = _pm1(rng, (7, 1, 1, 64))
    got = oracle.conv_pm1(x, f, 1, 0, -1)
    ref = oracle.dense_pm1(x.reshape(-1, 64), f.reshape(7, 64)).reshape(2, 4, 5, 7)
    assert np.array_equal(got, ref)


def test_conv_all_plus_one_closed_form():
    # 3x3, pad 1 treated as -1 (Sec. 5.2 "Zero-padding"): (inside taps - border taps) * C.
    C = 8
    x = np.ones((1, 4, 5, C), dtype=np.int8)
    f = np.ones((2, 3, 3, C), dtype=np.int8)
    out = oracle.conv_pm1(x, f, 1, 1, -1)
    assert out[0, 1, 1, 0] == 9 * C and out[0, 2, 3, 1] == 9 * C      # interior
    assert out[0, 0, 2, 0] == 3 * C and out[0, 2, 0, 0] == 3 * C      # edges: 6 in, 3 out
    for (m, n) in ((0, 0), (0, 4), (3, 0), (3, 4)):                     # corners: 4 in, 5 out
        assert out[0, m, n, 0] == -C


def test_conv_zero_padding_correction_identity():
    # Sec. 5.2 "Zero-padding for convolutions": the zero-padded convolution equals the
    # (-1)-padded one plus the convolution of the weights with a (+1)-padded zero tensor.
    rng = np.random.default_rng(12)
    x = _pm1(rng, (2, 6, 5, 16))
    f = _pm1(rng, (4, 3, 3, 16))
    zero_pad = oracle.conv_pm1(x, f, 1, 1, 0)
    minus_pad = oracle.conv_pm1(x, f, 1, 1, -1)
    correction = oracle.conv_pm1(np.zeros_like(x), f, 1, 1, +1)
    assert np.array_equal(zero_pad, minus_pad + correction)
    assert np.all(correction[:, 1:-1, 1:-1, :] == 0)     # only the border is touched
    assert np.any(correction != 0)


def test_unroll_then_dense_is_conv_and_layout():
    rng = np.random.default_rng(13)
    x = _pm1(rng, (2, 5, 4, 8))
    f = _pm1(rng, (3, 3, 3, 8))
    low = oracle.unroll_pm1(x, 3, 3, 1, 1, -1)
    assert low.shape == (2 * 5 * 4, 3 * 3 * 8)
    # Fig. 3: row (b*H2+m)*W2+n holds x[b, m-1:m+2, n-1:n+2, :] tap by tap.
    b, m, n = 1, 2, 1
    row = low[(b * 5 + m) * 4 + n].reshape(3, 3, 8)
    assert np.array_equal(row, x[b, m - 1:m + 2, n - 1:n + 2, :])
    corner = low[0].reshape(3, 3, 8)
    assert np.all(corner[0] == -1) and np.all(corner[:, 0] == -1)
    assert np.array_equal(corner[1:, 1:], x[0, 0:2, 0:2, :])
    out = oracle.dense_pm1(low, f.reshape(3, -1)).reshape(2, 5, 4, 3)
    assert np.array_equal(out, oracle.conv_pm1(x, f, 1, 1, -1))


def test_conv_library_third_opinion():
    rng = np.random.default_rng(14)
    x = _pm1(rng, (2, 7, 6, 5))
    f = _pm1(rng, (4, 3, 3, 5))
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    ft = torch.from_numpy(f.astype(np.float64)).permute(0, 3, 1, 2)
    for stride in (1, 2):
        xp = torch.nn.functional.pad(xt, (1, 1, 1, 1), value=-1.0)
        ref = torch.nn.functional.conv2d(xp, ft, stride=stride).permute(0, 2, 3, 1).numpy()
        assert np.array_equal(oracle.conv_pm1(x, f, stride, 1, -1), ref.astype(np.int32))


# ------------------------------------------------------------------ batch norm
def test_bn_special_cases():
    # var + eps = 1 exactly (0.75 + 0.25): y = gamma * (x - mean) + beta.
    assert oracle.bn_value(5.0, 2.0, -1.0, 3.0, 0.75, 0.25) == 3.0
    # var + eps = 4: divide by 2.  A dropped eps would divide by sqrt(3.75).
    assert oracle.bn_value(7.0, 3.0, 0.5, 1.0, 3.75, 0.25) == 9.5
    # x == mean gives beta whatever the rest.
    assert oracle.bn_value(-2.0, 17.0, 0.125, -2.0, 1.3, 1e-4) == 0.125
    # gamma < 0 flips the slope; gamma == 0 leaves beta.
    assert oracle.bn_value(4.0, -1.0, 0.0, 1.0, 0.75, 0.25) == -3.0
    assert oracle.bn_value(4.0, 0.0, -0.5, 1.0, 0.75, 0.25) == -0.5


def test_bn_array_per_channel_last_dim():
    x = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.int32)
    gamma = np.array([1, 2, -1], dtype=np.float32)
    beta = np.array([0, 1, 0.5], dtype=np.float32)
    mean = np.array([1, 0, 3], dtype=np.float32)
    var = np.array([0.75, 3.75, 0.75], dtype=np.float32)
    y = oracle.bn(x, gamma, beta, mean, var, 0.25)
    assert y.tolist() == [[0.0, 3.0, 0.5], [3.0, 6.0, -2.5]]
    assert np.array_equal(oracle.bn(x.astype(np.float64), gamma, beta, mean, var, 0.25), y)
    assert oracle.sign(y).tolist() == [[1, 1, 1], [1, 1, -1]]


def test_bn_matches_numpy_double_on_random_parameters():
    rng = np.random.default_rng(20)
    g, b, m, v = synth.bn_params(rng, 64)
    x = rng.integers(-1152, 1153, size=(50, 64)).astype(np.int32)
    eps = np.float32(1e-4)
    d = x.astype(np.float64) - m.astype(np.float64)
    ref = (g.astype(np.float64) * d) / np.sqrt(v.astype(np.float64) + np.float64(eps)) + b.astype(np.float64)
    assert np.array_equal(oracle.bn(x, g, b, m, v, float(eps)), ref)


# ------------------------------------------------------------------ max-pool
def test_maxpool_all_window_patterns():
    # Max of four +-1 values is +1 unless all four are -1 (the OR of the sign bits).
    pats = list(itertools.product((-1, 1), repeat=4))
    x = np.empty((1, 2, 2 * len(pats), 1), dtype=np.int8)
    for i, p in enumerate(pats):
        x[0, 0, 2 * i, 0], x[0, 0, 2 * i + 1, 0], x[0, 1, 2 * i, 0], x[0, 1, 2 * i + 1, 0] = p
    out = oracle.maxpool_pm1(x, 2, 2)
    assert out.shape == (1, 1, len(pats), 1)
    for i, p in enumerate(pats):
        assert out[0, 0, i, 0] == (1 if any(v == 1 for v in p) else -1)


def test_maxpool_library_third_opinion_and_floor():
    rng = np.random.default_rng(21)
    x = _pm1(rng, (2, 7, 6, 5))   # odd height: last row dropped
    out = oracle.maxpool_pm1(x, 2, 2)
    assert out.shape == (2, 3, 3, 5)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float32)).permute(0, 3, 1, 2), 2, 2)
    assert np.array_equal(out, ref.permute(0, 2, 3, 1).numpy().astype(np.int8))


@pytest.mark.parametrize("win,stride", [(3, 1), (3, 2), (3, 3), (2, 1), (4, 3)])
def test_maxpool_window_differs_from_stride(win, stride):
    # Pooling layer of Sec. 5.2 with a window that is not the stride: the window origin moves by
    # `stride`, its extent is `win`, and the output size is floor((size - win) / stride) + 1.
    # Brute force in numpy on a non-square input with odd sizes, then torch's max_pool2d as a
    # third opinion.  A mistake that swaps the two parameters anywhere changes a value or the shape.
    rng = np.random.default_rng(210 + 10 * win + stride)
    x = _pm1(rng, (2, 9, 11, 3))
    out = oracle.maxpool_pm1(x, win, stride)
    H2, W2 = (9 - win) // stride + 1, (11 - win) // stride + 1
    assert out.shape == (2, H2, W2, 3)
    ref = np.empty((2, H2, W2, 3), dtype=np.int8)
    for m in range(H2):
        for n in range(W2):
            ref[:, m, n, :] = x[:, m * stride:m * stride + win, n * stride:n * stride + win, :].max(axis=(1, 2))
    assert np.array_equal(out, ref)
    lib = torch.nn.functional.max_pool2d(torch.from_numpy(x.astype(np.float32)).permute(0, 3, 1, 2), win, stride)
    assert np.array_equal(out, lib.permute(0, 2, 3, 1).numpy().astype(np.int8))


def test_maxpool_single_plus_one_marks_exactly_the_windows_that_hold_it():
    # One +1 in a field of -1: output (m, n) is +1 exactly when m*stride <= y < m*stride + win and
    # n*stride <= x < n*stride + win (closed form, no library).
    for win, stride, y, x in ((3, 1, 4, 5), (3, 2, 4, 6), (2, 1, 3, 7), (3, 3, 5, 2)):
        a = -np.ones((1, 8, 10, 1), dtype=np.int8)
        a[0, y, x, 0] = 1
        out = oracle.maxpool_pm1(a, win, stride)
        H2, W2 = (8 - win) // stride + 1, (10 - win) // stride + 1
        assert out.shape == (1, H2, W2, 1)
        for m in range(H2):
            for n in range(W2):
                inside = m * stride <= y < m * stride + win and n * stride <= x < n * stride + win
                assert out[0, m, n, 0] == (1 if inside else -1), (win, stride, m, n)


# ------------------------------------------------------------------ float first layer
def test_float_dense_and_conv_against_library():
    rng = np.random.default_rng(22)
    x = rng.random((5, 37), dtype=np.float32)
    w = _pm1(rng, (11, 37))
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    np.testing.assert_allclose(oracle.dense_f64(x, w), ref, rtol=1e-13, atol=1e-13)
    # exactly representable case: inputs that are multiples of 1/8
    xe = (rng.integers(0, 9, size=(3, 20)) / 8.0).astype(np.float32)
    we = _pm1(rng, (4, 20))
    assert np.array_equal(oracle.dense_f64(xe, we), xe.astype(np.float64) @ we.astype(np.float64).T)

    img = rng.random((2, 6, 5, 3), dtype=np.float32)
    f = _pm1(rng, (4, 3, 3, 3))
    ref = torch.nn.functional.conv2d(torch.from_numpy(img.astype(np.float64)).permute(0, 3, 1, 2),
                                     torch.from_numpy(f.astype(np.float64)).permute(0, 3, 1, 2),
                                     padding=1).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(oracle.conv_f64(img, f, 1, 1), ref, rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------ fixed-precision first layer
def test_u8_first_layer_against_library_and_eq3_bitplanes():
    rng = np.random.default_rng(23)
    x = rng.integers(0, 256, size=(4, 37), dtype=np.uint8)
    x[0, :5] = [0, 255, 1, 128, 254]
    w = _pm1(rng, (6, 37))
    got = oracle.dense_u8(x, w)
    assert np.array_equal(got, x.astype(np.int64) @ w.astype(np.int64).T)
    # hand example: x = (3, 0, 255), w = (+, -, -): 3 - 0 - 255
    assert oracle.dense_u8(np.array([[3, 0, 255]], dtype=np.uint8),
                           np.array([[1, -1, -1]], dtype=np.int8)).tolist() == [[-252]]
    # Eq. 3: the product is the weighted sum of the products of the 0/1 bit-planes
    planes = [((x >> i) & 1).astype(np.int8) for i in range(8)]
    eq3 = sum((1 << i) * oracle.dense_pm1(planes[i], w).astype(np.int64) for i in range(8))
    assert np.array_equal(got, eq3)
    # ... and each 0/1 plane product follows from the +-1 product of the plane read as +-1:
    # p.w = ((2p-1).w + sum(w)) / 2
    wsum = w.astype(np.int64).sum(axis=1)
    for i in range(8):
        pm = (2 * planes[i] - 1).astype(np.int8)
        assert np.array_equal(2 * oracle.dense_pm1(planes[i], w), oracle.dense_pm1(pm, w) + wsum[None, :])

    img = rng.integers(0, 256, size=(2, 6, 5, 3), dtype=np.uint8)
    f = _pm1(rng, (4, 3, 3, 3))
    ref = torch.nn.functional.conv2d(torch.from_numpy(img.astype(np.float64)).permute(0, 3, 1, 2),
                                     torch.from_numpy(f.astype(np.float64)).permute(0, 3, 1, 2),
                                     padding=1).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(oracle.conv_u8(img, f, 1, 1), ref.astype(np.int32))
    assert np.array_equal(oracle.conv_u8(img, f, 2, 0),
                          torch.nn.functional.conv2d(torch.from_numpy(img.astype(np.float64)).permute(0, 3, 1, 2),
                                                     torch.from_numpy(f.astype(np.float64)).permute(0, 3, 1, 2),
                                                     stride=2).permute(0, 2, 3, 1).numpy().astype(np.int32))


# ------------------------------------------------------------------ network shapes
def test_network_shapes_match_paper_footprints():
    # Sec. 6.2 / 6.3 print the float and packed footprints; the parameter counts of the
    # layer shapes used here must reproduce them (weights only; the paper's figures
    # include the small batch-norm vectors, hence the tolerance).
    rows = {}
    with open(os.path.join(GOLDEN, "paper_footprints.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, packed, full = line.split()
            rows[name] = (float(packed), float(full))
    mlp = sum(k * n for k, n in zip(synth.MLP_SIZES[:-1], synth.MLP_SIZES[1:]))
    assert mlp == 36806656
    cnn = 0
    for l in synth.CNN_LAYERS:
        if l[0] == "conv":
            cnn += 9 * l[1] * l[2]
        elif l[0] == "dense":
            cnn += l[1] * l[2]
    assert cnn == 14022016
    for name, count in (("mlp", mlp), ("cnn", cnn)):
        packed_mb, float_mb = rows[name]
        assert abs(count * 4 / 2**20 - float_mb) / float_mb < 0.005
        assert abs(count / 8 / 2**20 - packed_mb) / packed_mb < 0.05


def test_mlp_and_cnn_forward_chain_small():
    # The network oracles are plain chains of the layer oracles; check the chaining on
    # reduced shapes against an explicit re-chaining, and the flatten order.
    rng = np.random.default_rng(30)
    sizes = (12, 16, 16, 5)
    layers = []
    for i in range(3):
        layers.append({"w": _pm1(rng, (sizes[i + 1], sizes[i])),
                       "bn": synth.bn_params(rng, sizes[i + 1]) if i < 2 else None})
    x = rng.random((3, 12), dtype=np.float32)
    tr = nets.mlp_forward(x, layers, 1e-4)
    a1 = oracle.sign(oracle.bn(oracle.dense_f64(x, layers[0]["w"]), *layers[0]["bn"], 1e-4))
    a2 = oracle.sign(oracle.bn(oracle.dense_pm1(a1, layers[1]["w"]), *layers[1]["bn"], 1e-4))
    assert np.array_equal(tr[-1]["pre"], oracle.dense_pm1(a2, layers[2]["w"]))
    assert tr[-1]["pre"].dtype == np.int32 and tr[-1]["pre"].shape == (3, 5)

    spec = (("conv", 3, 8), ("conv", 8, 8), ("pool",), ("dense", 8 * 2 * 2, 6), ("dense", 6, 4))
    params = []
    for i, l in enumerate(spec):
        if l[0] == "pool":
            params.append({"kind": "pool"})
        elif l[0] == "conv":
            params.append({"kind": "conv", "w": _pm1(rng, (l[2], 3, 3, l[1])), "bn": synth.bn_params(rng, l[2])})
        else:
            params.append({"kind": "dense", "w": _pm1(rng, (l[2], l[1])),
                           "bn": synth.bn_params(rng, l[2]) if i < len(spec) - 1 else None})
    img = rng.random((2, 4, 4, 3), dtype=np.float32)
    tr = nets.cnn_forward(img, params, 1e-4)
    c1 = oracle.sign(oracle.bn(oracle.conv_f64(img, params[0]["w"], 1, 1), *params[0]["bn"], 1e-4))
    c2 = oracle.sign(oracle.bn(oracle.conv_pm1(c1, params[1]["w"], 1, 1, -1), *params[1]["bn"], 1e-4))
    p = oracle.maxpool_pm1(c2, 2, 2)
    d1 = oracle.sign(oracle.bn(oracle.dense_pm1(p.reshape(2, -1), params[3]["w"]), *params[3]["bn"], 1e-4))
    assert np.array_equal(tr[-1]["pre"], oracle.dense_pm1(d1, params[4]["w"]))
    # substituting the first activation restarts the chain from it
    tr2 = nets.cnn_forward(img, params, 1e-4, first_act=-c1)
    c2b = oracle.sign(oracle.bn(oracle.conv_pm1(-c1, params[1]["w"], 1, 1, -1), *params[1]["bn"], 1e-4))
    assert np.array_equal(tr2[1]["act"], c2b)
