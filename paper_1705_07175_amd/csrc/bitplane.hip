// Binary first layer on fixed-precision input (arXiv 1705.07175, Sec. 4.3, Eq. 3, and
// Sec. 6.2 "First-layer binary optimization"): an 8-bit input is split into its 8
// bit-planes, each plane goes through the ordinary packed XOR-popcount product, and the
// eight results are recombined by a weighted sum.
//
// The paper does not spell out how a {0,1}-valued plane enters a product defined on +-1
// values.  Here plane bit p is stored as it is (bit 1 = +1, bit 0 = -1 for the product),
// which yields d_i = sum_k (2 p_k - 1) w_k, and the recombination undoes the offset:
//   sum_k x_k w_k = sum_i 2^i sum_k p_ik w_k = ( sum_i 2^i d_i + 255 * sum_k w_k ) / 2,
// exact in integers (d_i and sum_k w_k have the parity of K).  A pixel of value 0 is all
// zero bits = -1 in every plane, which is exactly the -1 border of the binary convolution,
// so zero padding of the image needs no correction.
#include "esp_internal.h"

namespace esp {

// x [outer][inner][k] uint8 -> planes [outer][8][inner][Kw]: wave = one 64-value word of
// one (outer, inner) row; lane l reads byte 64*w + l, eight ballots give the eight words.
__global__ __launch_bounds__(256)
void bitplane_pack_kernel(const uint8_t *__restrict__ x, uint64_t *__restrict__ planes,
                          int64_t rows, int64_t inner, int k, int Kw)
{
    const int lane = threadIdx.x % kWave;
    const int64_t task = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (task >= rows * Kw)
        return;
    const int w = (int)(task % Kw);
    const int64_t row = task / Kw;
    const int64_t o = row / inner, in = row - o * inner;
    const int c = w * 64 + lane;
    const unsigned v = c < k ? x[row * k + c] : 0u;
    uint64_t mine = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint64_t word = __ballot((v >> i) & 1u);
        if (lane == i)
            mine = word;
    }
    if (lane < 8)
        planes[((o * 8 + lane) * inner + in) * Kw + w] = mine;
}

// wsum[n] = sum_k w[n][k] over the true K = 2 * popcount(row) - K.
__global__ __launch_bounds__(256)
void row_sums_kernel(const uint64_t *__restrict__ W, int32_t *__restrict__ wsum, int N, int K, int Kw)
{
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N)
        return;
    int ones = 0;
    for (int w = 0; w < Kw; ++w)
        ones += __popcll(W[(int64_t)n * Kw + w]);
    wsum[n] = 2 * ones - K;
}

// y[o][in][n] = ( sum_i 2^i d[o][i][in][n] + 255 * wsum[n] ) / 2
__global__ __launch_bounds__(256)
void bitplane_combine_kernel(const int32_t *__restrict__ d, const int32_t *__restrict__ wsum,
                             int32_t *__restrict__ y, int64_t outer, int64_t inner, int N)
{
    const int64_t total = outer * inner * N;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total)
        return;
    const int n = (int)(idx % N);
    const int64_t row = idx / N;
    const int64_t o = row / inner, in = row - o * inner;
    int64_t acc = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        acc += (int64_t)d[(((o * 8 + i) * inner) + in) * N + n] << i;
    acc += 255ll * wsum[n];
    y[idx] = (int32_t)(acc / 2);   // acc is even
}

} // namespace esp

extern "C" int esp_bitplane_pack_u8(const uint8_t *x, uint64_t *planes, int64_t outer, int64_t inner,
                                    int64_t k, esp_stream stream)
{
    using namespace esp;
    if (outer < 0 || inner <= 0 || k <= 0)
        return ESP_EINVAL;
    if (k >= kMaxK / 256)
        return ESP_ESHAPE;   // keeps 255 * K inside the int32 contract
    if (outer == 0)
        return ESP_OK;
    if (!x || !planes)
        return ESP_EINVAL;
    if (!aligned(planes, 8))
        return ESP_EALIGN;
    const int64_t Kw = ceil_div(k, 64);
    const int64_t tasks = outer * inner * Kw;
    hipLaunchKernelGGL(bitplane_pack_kernel, dim3(grid_for(tasks, 4)), dim3(256), 0, as_stream(stream), x,
                       planes, outer * inner, inner, (int)k, (int)Kw);
    return launch_status();
}

extern "C" int esp_row_sums(const uint64_t *W, int32_t *wsum, int64_t N, int64_t row_words, int64_t K,
                            esp_stream stream)
{
    using namespace esp;
    if (N <= 0 || K <= 0 || row_words <= 0)
        return ESP_EINVAL;
    if (K >= kMaxK || N >= (1ll << 31) || row_words >= (1ll << 29) || K > row_words * 64)
        return ESP_ESHAPE;
    if (!W || !wsum)
        return ESP_EINVAL;
    if (!aligned(W, 8) || !aligned(wsum, 4))
        return ESP_EALIGN;
    hipLaunchKernelGGL(row_sums_kernel, dim3(grid_for(N, 256)), dim3(256), 0, as_stream(stream), W, wsum,
                       (int)N, (int)K, (int)row_words);
    return launch_status();
}

extern "C" int esp_bitplane_combine(const int32_t *d, const int32_t *wsum, int32_t *y, int64_t outer,
                                    int64_t inner, int64_t N, esp_stream stream)
{
    using namespace esp;
    if (outer < 0 || inner <= 0 || N <= 0)
        return ESP_EINVAL;
    if (N >= (1ll << 31))
        return ESP_ESHAPE;
    if (outer == 0)
        return ESP_OK;
    if (!d || !wsum || !y)
        return ESP_EINVAL;
    if (!aligned(d, 4) || !aligned(wsum, 4) || !aligned(y, 4))
        return ESP_EALIGN;
    const int64_t total = outer * inner * N;
    hipLaunchKernelGGL(bitplane_combine_kernel, dim3(grid_for(total, 256)), dim3(256), 0, as_stream(stream),
                       d, wsum, y, outer, inner, (int)N);
    return launch_status();
}

extern "C" int esp_bitplane_dense(const uint64_t *planes, const uint64_t *W, const int32_t *wsum,
                                  const int32_t *thr, const uint64_t *flip, uint64_t *bits, int32_t *y,
                                  int64_t rows, int64_t N, int64_t K, esp_stream stream)
{
    using namespace esp;
    if (rows < 0 || N <= 0 || K <= 0)
        return ESP_EINVAL;
    if (K >= (1 << 21))
        return ESP_ESHAPE;
    if (rows == 0)
        return ESP_OK;
    if (!planes || !W || !wsum || (!bits && !y) || (bits && (!thr || !flip)))
        return ESP_EINVAL;
    if (!aligned(planes, 8) || !aligned(W, 8) || !aligned(wsum, 4) || !aligned(thr, 4) || !aligned(flip, 8) ||
        !aligned(bits, 8) || !aligned(y, 4))
        return ESP_EALIGN;
    return bitplane_dense_mfma_launch(planes, W, wsum, y, thr, flip, bits, rows, N, K, ceil_div(K, 64),
                                      as_stream(stream));
}
