"""GPU parity at the sizes and launch shapes that bench.py times for the bandwidth-bound
supporting kernels (1 GiB-class inputs).  The oracle cannot redo a whole 1 GiB array in
seconds, so it recomputes sampled rows / images one by one, always including the first and the
last (the edges of the grid) and a few seeded ones in between; the GPU result must be
identical there.  Inputs are seeded torch draws on the device; the sampled parts are copied
to the host for the oracle."""
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


def _gen(seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(synth.SEED0 + seed)
    return g


def _rand_words(shape, g):
    return torch.randint(-2**62, 2**62, shape, device=DEV, generator=g, dtype=torch.int64)


def _sample(n, k, seed):
    rng = np.random.default_rng(seed)
    return np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, k)]))


def _words_np(t):
    return t.cpu().numpy().view(np.uint64)


def test_pack_f32_1gib():
    rows, k = 16384, 16384
    x = torch.rand((rows, k), device=DEV, generator=_gen(1)) - 0.5
    out = esp.pack_f32(x)
    idx = _sample(rows, 6, 1)
    xs = x[torch.from_numpy(idx).to(DEV)].cpu().numpy()
    assert np.array_equal(_words_np(out[torch.from_numpy(idx).to(DEV)]), oracle.pack_bits(oracle.sign(xs)))


def test_bn_sign_pack_1gib():
    rows, c = 2 * 1024 * 1024, 128
    x = torch.randint(-1152, 1153, (rows, c), device=DEV, generator=_gen(2), dtype=torch.int32)
    bnp = synth.bn_params(np.random.default_rng(2), c)
    bnp = (bnp[0], bnp[1], (bnp[2] * 30).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    out = esp.bn_sign_pack(x, torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV))
    idx = torch.from_numpy(_sample(rows, 30, 2)).to(DEV)
    want = oracle.pack_bits(oracle.bn_sign(x[idx].cpu().numpy(), bnp, synth.BN_EPS))
    assert np.array_equal(_words_np(out[idx]), want)


def test_unroll_576mib():
    b, h, c = 4096, 32, 128
    x = _rand_words((b, h, h, c // 64), _gen(3))
    low = esp.unroll(x, c, 3, 3, 1, 1)
    assert low.shape == (b * h * h, 9 * c // 64)
    for img in _sample(b, 2, 3):
        xi = oracle.unpack_bits(_words_np(x[int(img)]), c)[None]            # [1][32][32][128] +-1
        want = oracle.pack_bits(oracle.unroll_pm1(xi, 3, 3, 1, 1, -1).reshape(h * h, 9, c))
        got = _words_np(low[int(img) * h * h:(int(img) + 1) * h * h])
        assert np.array_equal(got, want.reshape(h * h, -1)), img


def test_bmaxpool_1gib():
    b, h, c = 4096, 64, 512
    x = _rand_words((b, h, h, c // 64), _gen(4))
    out = esp.bmaxpool(x, c, 2, 2)
    for img in _sample(b, 2, 4):
        xi = oracle.unpack_bits(_words_np(x[int(img)]), c)[None]
        want = oracle.pack_bits(oracle.maxpool_pm1(xi, 2, 2))[0]
        assert np.array_equal(_words_np(out[int(img)]), want), img


@pytest.mark.parametrize("nrows", [16384, 524288])
def test_bgemv_bench_shapes(nrows):
    # config 5's matrix-vector product (32 MiB of weights) and the 1 GiB variant bench.py times
    k = 16384
    g = _gen(5)
    w = _rand_words((nrows, k // 64), g)
    a = _rand_words((1, k // 64), g)
    c = esp.bgemm(a, w, k)
    idx = _sample(nrows, 40, 5)
    ws = oracle.unpack_bits(_words_np(w[torch.from_numpy(idx).to(DEV)]), k)
    av = oracle.unpack_bits(_words_np(a), k)
    assert np.array_equal(c.cpu().numpy()[0, idx], oracle.dense_pm1(av, ws)[0])
    # every output has the parity of K and lies in [-K, K]
    cn = c.cpu().numpy()
    assert cn.min() >= -k and cn.max() <= k and not np.any((cn - k) & 1)


def test_conv1_batch256_sampled_images():
    # the real-valued first convolution at the batch bench.py times (fp32 matrix-core kernel)
    b, h, l2 = 256, 32, 128
    layers = synth.cnn_params()
    x = synth.cnn_input(b)
    f = layers[0]["w"]
    thr, sgn = esp.bn_fold_f32(*layers[0]["bn"], synth.BN_EPS)
    pre = torch.empty((b, h, h, l2), dtype=torch.float32, device=DEV)
    bits = esp.conv_f32_bn_sign_pack(torch.from_numpy(x).to(DEV), torch.from_numpy(f.astype(np.float32)).to(DEV),
                                     torch.from_numpy(thr).to(DEV), torch.from_numpy(sgn).to(DEV), 1, 1, pre=pre)
    idx = _sample(b, 2, 6)
    ref = oracle.conv_f64(x[idx], f, 1, 1)
    got = pre.cpu().numpy()[idx]
    assert np.all(np.abs(got - ref) <= 1e-4 * np.maximum(1.0, np.abs(ref)))
    want_bits = oracle.pack_bits(oracle.bn_sign(got.astype(np.float64), layers[0]["bn"], synth.BN_EPS))
    assert np.array_equal(_words_np(bits)[idx], want_bits)


# ---- beyond 2^31 elements: element offsets no longer fit 32 bits -------------------------------
def test_bgemm_output_beyond_2_to_31_elements():
    # C has 140000 x 16384 = 2.29e9 int32 values (9.2 GB); K = 64 keeps the product itself small
    M, N, K = 140000, 16384, 64
    g = _gen(20)
    A = _rand_words((M, 1), g)
    B = _rand_words((N, 1), g)
    C = esp.bgemm(A, B, K)
    rows = _sample(M, 6, 20)
    a = oracle.unpack_bits(_words_np(A[torch.from_numpy(rows).to(DEV)]), K)
    b = oracle.unpack_bits(_words_np(B), K)
    assert np.array_equal(C[torch.from_numpy(rows).to(DEV)].cpu().numpy(), oracle.dense_pm1(a, b))
    del C
    torch.cuda.empty_cache()


def test_pack_f32_beyond_2_to_31_elements():
    rows, k = 70000, 32768           # 2.29e9 floats (9.2 GB)
    x = torch.rand((rows, k), device=DEV, generator=_gen(21)) - 0.5
    out = esp.pack_f32(x)
    idx = _sample(rows, 5, 21)
    xs = x[torch.from_numpy(idx).to(DEV)].cpu().numpy()
    assert np.array_equal(_words_np(out[torch.from_numpy(idx).to(DEV)]), oracle.pack_bits(oracle.sign(xs)))
    del x, out
    torch.cuda.empty_cache()


def test_bn_sign_pack_beyond_2_to_31_elements():
    rows, c = 18 * 1024 * 1024, 128  # 2.42e9 int32 values (9.7 GB)
    x = torch.randint(-1152, 1153, (rows, c), device=DEV, generator=_gen(22), dtype=torch.int32)
    bnp = synth.bn_params(np.random.default_rng(22), c)
    bnp = (bnp[0], bnp[1], (bnp[2] * 30).astype(np.float32), bnp[3])
    thr, flip = esp.bn_fold(*bnp, synth.BN_EPS)
    out = esp.bn_sign_pack(x, torch.from_numpy(thr).to(DEV), esp.to_packed_tensor(flip, DEV))
    idx = _sample(rows, 6, 22)
    xs = x[torch.from_numpy(idx).to(DEV)].cpu().numpy()
    assert np.array_equal(_words_np(out[torch.from_numpy(idx).to(DEV)]), oracle.pack_bits(oracle.bn_sign(xs, bnp, synth.BN_EPS)))
    del x, out
    torch.cuda.empty_cache()


def test_bgemm_mfma_output_beyond_2_to_31_elements():
    M, N, K = 140000, 16384, 128
    g = _gen(23)
    A = _rand_words((M, 2), g)
    B = _rand_words((N, 2), g)
    C = esp.bgemm_mfma(A, B, K)
    rows = _sample(M, 6, 23)
    a = oracle.unpack_bits(_words_np(A[torch.from_numpy(rows).to(DEV)]), K)
    b = oracle.unpack_bits(_words_np(B), K)
    assert np.array_equal(C[torch.from_numpy(rows).to(DEV)].cpu().numpy(), oracle.dense_pm1(a, b))
    del C
    torch.cuda.empty_cache()
