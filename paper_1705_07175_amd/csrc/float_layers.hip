// Real-valued first layer in fp32 (the non-binary variant of a layer, Sec. 3 of
// arXiv 1705.07175): the networks of Sec. 6.2 / 6.3 start from real-valued images, so
// their first dense / convolutional layer multiplies floats by +-1 weights.  These are
// supporting kernels, kept simple: an LDS-tiled SGEMM, a wave-per-output GEMV for tiny
// batches and a direct convolution with the filters transposed in LDS.
#include "esp_internal.h"

namespace esp {

// Y[M][N] = X[M][K] * W[N][K]^T, 64x64 tile, 256 threads, 4x4 outputs per thread.
__global__ __launch_bounds__(256)
void dense_f32_tile_kernel(const float *__restrict__ X, const float *__restrict__ Wt,
                           float *__restrict__ Y, int M, int N, int K)
{
    constexpr int BT = 64, BK = 16;
    __shared__ float Xs[BK][BT + 4];
    __shared__ float Ws[BK][BT + 4];
    const int tid = threadIdx.x;
    const int tx = tid % 16, ty = tid / 16;
    const int m0 = blockIdx.y * BT, n0 = blockIdx.x * BT;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        // 64 rows x 16 k per operand = 1024 values, 4 per thread; k fastest so that a
        // group of 16 lanes reads 64 contiguous bytes of one row
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + i * 256;
            const int r = idx / BK, k = idx % BK;
            const bool kin = k0 + k < K;
            Xs[k][r] = (kin && m0 + r < M) ? X[(int64_t)(m0 + r) * K + k0 + k] : 0.0f;
            Ws[k][r] = (kin && n0 + r < N) ? Wt[(int64_t)(n0 + r) * K + k0 + k] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = Xs[k][ty + 16 * i];
                b[i] = Ws[k][tx + 16 * i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty + 16 * i;
        if (m >= M)
            continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx + 16 * j;
            if (n < N)
                Y[(int64_t)m * N + n] = acc[i][j];
        }
    }
}

// Small batch: one wave per output neuron n, lanes stride over K, all (<= 4) rows of X
// reuse each weight load; butterfly sum at the end.
template <int MS>
__global__ __launch_bounds__(256)
void dense_f32_gemv_kernel(const float *__restrict__ X, const float *__restrict__ Wt,
                           float *__restrict__ Y, int M, int N, int K)
{
    const int lane = threadIdx.x % kWave;
    const int64_t n = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (n >= N)
        return;
    float acc[MS];
#pragma unroll
    for (int m = 0; m < MS; ++m)
        acc[m] = 0.0f;
    const float *wrow = Wt + n * K;
    for (int k = lane; k < K; k += kWave) {
        const float w = wrow[k];
#pragma unroll
        for (int m = 0; m < MS; ++m)
            if (m < M)
                acc[m] = fmaf(X[(int64_t)m * K + k], w, acc[m]);
    }
#pragma unroll
    for (int m = 0; m < MS; ++m) {
        float v = acc[m];
        for (int off = 32; off > 0; off >>= 1)
            v += __shfl_xor(v, off, kWave);
        if (lane == 0 && m < M)
            Y[(int64_t)m * N + n] = v;
    }
}

// Direct NHWC convolution, zero padding.  The block copies the filters to LDS as
// [tap*C + c][L2] so that lanes (= output channels) read consecutive addresses, then
// walks its share of output pixels; the input value of a tap is the same for every lane
// of a pixel.
__global__ __launch_bounds__(256)
void conv_f32_kernel(const float *__restrict__ in, const float *__restrict__ filt,
                     float *__restrict__ out, int B, int H, int W, int C, int L2, int kh, int kw,
                     int stride, int pad, int H2, int W2, int filt_in_lds)
{
    extern __shared__ float fT[];
    const int taps = kh * kw * C;
    if (filt_in_lds) {
        for (int i = threadIdx.x; i < taps * L2; i += blockDim.x) {
            const int l2 = i / taps, t = i % taps;
            fT[t * L2 + l2] = filt[i];
        }
        __syncthreads();
    }
    const int64_t total = (int64_t)B * H2 * W2 * L2;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total; o += step) {
        const int l2 = (int)(o % L2);
        const int64_t pix = o / L2;
        const int n = (int)(pix % W2);
        const int m = (int)((pix / W2) % H2);
        const int b = (int)(pix / ((int64_t)W2 * H2));
        float acc = 0.0f;
        for (int dy = 0; dy < kh; ++dy) {
            const int y = m * stride + dy - pad;
            if (y < 0 || y >= H)
                continue;
            for (int dx = 0; dx < kw; ++dx) {
                const int x = n * stride + dx - pad;
                if (x < 0 || x >= W)
                    continue;
                const float *ip = in + (((int64_t)b * H + y) * W + x) * C;
                const int t0 = (dy * kw + dx) * C;
                for (int c = 0; c < C; ++c) {
                    const float f = filt_in_lds ? fT[(t0 + c) * L2 + l2] : filt[(int64_t)l2 * taps + t0 + c];
                    acc = fmaf(ip[c], f, acc);
                }
            }
        }
        out[o] = acc;
    }
}

// Fast path for small, compile-time filter shapes at stride 1 (the 3x3x3 first layer of the
// Sec. 6.3 network): lane = output channel with its KH*KW*C filter weights in registers; a
// wave owns a strip of PIX consecutive output pixels of one output row.  The wave first
// copies the strip's input window (KH rows x (PIX+KW-1) pixels x C, zeros outside the image)
// into its private LDS slice, then every lane reads the whole window back with broadcast
// 16-byte LDS reads, so the inner loop is KH*KW*C register-to-register fused multiply-adds
// per output with no address arithmetic.  The 64 lanes store 256 contiguous bytes per pixel.
// A wave walks all strips of its output row, so the weights are fetched once per row.
// With FUSE the folded batch-norm threshold + sign is applied in the epilogue: the 64-lane
// comparison mask of a pixel is its packed word, so only bits leave the kernel (the
// pre-activations are written as well only if `out` is given).
template <int C, int KH, int KW, int PIX, bool FUSE>
__global__ __launch_bounds__(256)
void conv_f32_lane_channel_kernel(const float *__restrict__ in, const float *__restrict__ filt,
                                  float *__restrict__ out, const float *__restrict__ thr,
                                  const float *__restrict__ sgn, uint64_t *__restrict__ bits,
                                  int H, int W, int L2, int pad, int H2, int W2, int cgroups, int tasks)
{
    constexpr int T = KH * KW * C;
    constexpr int RL = (PIX + KW - 1) * C;          // floats per window row
    constexpr int RLP = (RL + 3) / 4 * 4;           // padded to whole float4s
    constexpr int WIN = KH * RLP;
    __shared__ __align__(16) float win_all[4][WIN];

    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int task = blockIdx.x * (blockDim.x / kWave) + wave;   // wave-uniform
    if (task >= tasks)
        return;
    // task -> (image row bm = b*H2 + m, channel group); channel group fastest
    const int cg = task % cgroups;
    const int bm = task / cgroups;
    const int m = bm % H2;
    const int b = bm / H2;
    const int l2 = cg * kWave + lane;
    const bool lane_ok = l2 < L2;

    float wgt[T];
#pragma unroll
    for (int t = 0; t < T; ++t)
        wgt[t] = lane_ok ? filt[l2 * T + t] : 0.0f;

    float th = 0.0f, sg = 1.0f;
    if (FUSE && lane_ok) {
        th = thr[l2];
        sg = sgn[l2];
    }

    float *win = win_all[wave];
    const float *img = in + (int64_t)b * H * W * C;
    float *orow = out + ((int64_t)bm * W2) * L2 + l2;
    for (int n0 = 0; n0 < W2; n0 += PIX) {
    uint64_t mine = 0;
    // window -> LDS (zero padding applied here)
    for (int i = lane; i < WIN; i += kWave) {
        const int r = i / RLP, j = i % RLP;
        const int y = m - pad + r;
        const int x = n0 - pad + j / C;
        float v = 0.0f;
        if (j < RL && y >= 0 && y < H && x >= 0 && x < W)
            v = img[(y * W + x) * C + j % C];
        win[i] = v;
    }
    // LDS operations of one wave complete in order: no barrier needed for a private slice
    float wv[WIN];
#pragma unroll
    for (int q = 0; q < WIN / 4; ++q) {
        const float4 t4 = *reinterpret_cast<const float4 *>(win + 4 * q);
        wv[4 * q + 0] = t4.x;
        wv[4 * q + 1] = t4.y;
        wv[4 * q + 2] = t4.z;
        wv[4 * q + 3] = t4.w;
    }

#pragma unroll
    for (int p = 0; p < PIX; ++p) {
        float acc = 0.0f;
#pragma unroll
        for (int dy = 0; dy < KH; ++dy)
#pragma unroll
            for (int dx = 0; dx < KW; ++dx)
#pragma unroll
                for (int c = 0; c < C; ++c)
                    acc = fmaf(wv[dy * RLP + (p + dx) * C + c], wgt[(dy * KW + dx) * C + c], acc);
        if ((!FUSE || out) && lane_ok && n0 + p < W2)
            orow[(int64_t)(n0 + p) * L2] = acc;
        if (FUSE) {
            const uint64_t word = __ballot(lane_ok && sg * acc >= th);
            if (lane == p)
                mine = word;
        }
    }
    if (FUSE && lane < PIX && n0 + lane < W2)
        bits[((int64_t)bm * W2 + n0 + lane) * cgroups + cg] = mine;
    } // strips
}

} // namespace esp

extern "C" int esp_dense_f32(const float *X, const float *W, float *Y,
                             int64_t M, int64_t N, int64_t K, esp_stream stream)
{
    using namespace esp;
    if (M < 0 || N <= 0 || K <= 0)
        return ESP_EINVAL;
    if (M >= (1ll << 31) || N >= (1ll << 31) || K >= (1ll << 31))
        return ESP_ESHAPE;
    if (M == 0)
        return ESP_OK;
    if (!X || !W || !Y)
        return ESP_EINVAL;
    if (!aligned(X, 4) || !aligned(W, 4) || !aligned(Y, 4))
        return ESP_EALIGN;
    hipStream_t s = as_stream(stream);
    if (M <= 4) {
        const dim3 grid((unsigned)ceil_div(N, 4));
        if (M == 1)
            hipLaunchKernelGGL((dense_f32_gemv_kernel<1>), grid, dim3(256), 0, s, X, W, Y, (int)M, (int)N, (int)K);
        else
            hipLaunchKernelGGL((dense_f32_gemv_kernel<4>), grid, dim3(256), 0, s, X, W, Y, (int)M, (int)N, (int)K);
        return launch_status();
    }
    const int64_t gy = ceil_div(M, 64);
    if (gy > 65535)
        return ESP_ESHAPE;
    const dim3 grid((unsigned)ceil_div(N, 64), (unsigned)gy);
    hipLaunchKernelGGL(dense_f32_tile_kernel, grid, dim3(256), 0, s, X, W, Y, (int)M, (int)N, (int)K);
    return launch_status();
}

namespace esp {

static int conv_f32_launch(const float *in, const float *filt, float *out, const float *thr,
                           const float *sgn, uint64_t *bits, int B, int H, int W, int C, int L2,
                           int kh, int kw, int stride, int pad, hipStream_t stream, bool *done)
{
    // fast path: 3x3x3 filters at stride 1 (the first layer of the Sec. 6.3 network)
    *done = false;
    const int H2 = (H + 2 * pad - kh) / stride + 1;
    const int W2 = (W + 2 * pad - kw) / stride + 1;
    if (!(C == 3 && kh == 3 && kw == 3 && stride == 1 && (int64_t)H * W * C < (1ll << 31) &&
          (int64_t)L2 * 27 < (1ll << 31)))
        return ESP_OK;
    constexpr int PIX = 8;
    const int cgroups = (L2 + kWave - 1) / kWave;
    const int64_t tasks = (int64_t)B * H2 * cgroups;
    if (tasks >= (1ll << 31))
        return ESP_OK;
    *done = true;
    if (bits)
        hipLaunchKernelGGL((conv_f32_lane_channel_kernel<3, 3, 3, PIX, true>), dim3(grid_for(tasks, 4)),
                           dim3(256), 0, stream, in, filt, out, thr, sgn, bits, H, W, L2, pad, H2, W2,
                           cgroups, (int)tasks);
    else
        hipLaunchKernelGGL((conv_f32_lane_channel_kernel<3, 3, 3, PIX, false>), dim3(grid_for(tasks, 4)),
                           dim3(256), 0, stream, in, filt, out, thr, sgn, bits, H, W, L2, pad, H2, W2,
                           cgroups, (int)tasks);
    return launch_status();
}

static int conv_f32_args(const float *in, const float *filt, int B, int H, int W, int C, int L2,
                         int kh, int kw, int stride, int pad)
{
    if (B < 0 || H <= 0 || W <= 0 || C <= 0 || L2 <= 0 || kh <= 0 || kw <= 0)
        return ESP_EINVAL;
    if (stride < 1 || pad < 0 || (int64_t)H + 2 * (int64_t)pad < kh || (int64_t)W + 2 * (int64_t)pad < kw)
        return ESP_ESHAPE;
    if (B == 0)
        return ESP_OK;
    if (!in || !filt)
        return ESP_EINVAL;
    if (!aligned(in, 4) || !aligned(filt, 4))
        return ESP_EALIGN;
    return ESP_OK;
}

static int conv_f32_generic(const float *in, const float *filt, float *out, int B, int H, int W, int C,
                            int L2, int kh, int kw, int stride, int pad, hipStream_t stream)
{
    const int H2 = (H + 2 * pad - kh) / stride + 1;
    const int W2 = (W + 2 * pad - kw) / stride + 1;
    const int64_t total = (int64_t)B * H2 * W2 * L2;
    const size_t lds = (size_t)kh * kw * C * L2 * sizeof(float);
    const int in_lds = lds <= 48 * 1024;
    const unsigned grid = grid_for(total, 256 * 8, 256 * 64);
    hipLaunchKernelGGL(conv_f32_kernel, dim3(grid), dim3(256), in_lds ? lds : 0, stream, in, filt, out, B,
                       H, W, C, L2, kh, kw, stride, pad, H2, W2, in_lds);
    return launch_status();
}

} // namespace esp

extern "C" int esp_conv_f32(const float *in, const float *filt, float *out,
                            int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                            esp_stream stream)
{
    using namespace esp;
    const int st = conv_f32_args(in, filt, B, H, W, C, L2, kh, kw, stride, pad);
    if (st != ESP_OK || B == 0)
        return st;
    if (!out)
        return ESP_EINVAL;
    if (!aligned(out, 4))
        return ESP_EALIGN;
    bool done;
    const int fs = conv_f32_launch(in, filt, out, nullptr, nullptr, nullptr, B, H, W, C, L2, kh, kw,
                                   stride, pad, as_stream(stream), &done);
    if (done)
        return fs;
    return conv_f32_generic(in, filt, out, B, H, W, C, L2, kh, kw, stride, pad, as_stream(stream));
}

extern "C" int esp_conv_f32_bn_sign_pack(const float *in, const float *filt, const float *thr,
                                         const float *sgn, uint64_t *bits, float *pre,
                                         int B, int H, int W, int C, int L2, int kh, int kw, int stride,
                                         int pad, esp_stream stream)
{
    using namespace esp;
    const int st = conv_f32_args(in, filt, B, H, W, C, L2, kh, kw, stride, pad);
    if (st != ESP_OK || B == 0)
        return st;
    if (!thr || !sgn || !bits)
        return ESP_EINVAL;
    if (!aligned(thr, 4) || !aligned(sgn, 4) || !aligned(bits, 8) || (pre && !aligned(pre, 4)))
        return ESP_EALIGN;
    bool done;
    const int fs = conv_f32_launch(in, filt, pre, thr, sgn, bits, B, H, W, C, L2, kh, kw, stride, pad,
                                   as_stream(stream), &done);
    if (done)
        return fs;
    // other filter shapes: the two-kernel route needs the pre-activation buffer
    if (!pre)
        return ESP_EWORKSPACE;
    const int cs = conv_f32_generic(in, filt, pre, B, H, W, C, L2, kh, kw, stride, pad, as_stream(stream));
    if (cs != ESP_OK)
        return cs;
    const int64_t H2 = (H + 2 * pad - kh) / stride + 1;
    const int64_t W2 = (W + 2 * pad - kw) / stride + 1;
    return esp_bn_sign_pack_f32(pre, thr, sgn, bits, (int64_t)B * H2 * W2, L2, stream);
}
