// Real-valued first layer (the non-binary variant of a layer, Sec. 3 of
// arXiv 1705.07175): the networks of Sec. 6.2 / 6.3 start from real-valued images, so
// their first dense / convolutional layer multiplies floats by +-1 weights.  These are
// supporting kernels: LDS-tiled dense layers on the matrix cores (fp32 operands for the plain
// product, three exact bf16 terms per input for the fused layer), a wave-per-output GEMV for
// tiny batches, a direct convolution with the filters transposed in LDS for general shapes,
// and the 3x3x3 first layer of the CIFAR-10 network on the bf16 matrix cores (three exact
// terms per input as well).
#include "esp_internal.h"

namespace esp {

// Y[M][N] = X[M][K] * W[N][K]^T on the fp32 matrix cores (v_mfma_f32_32x32x2_f32): 64 x BN
// block tile, 256 threads = 4 waves, K in slabs of 32 staged in LDS k-major, so that lane
// (row or column lane % 32, k half lane / 32) reads its A and B operand of a k-step with one
// conflict-free 4-byte LDS read each.  BN = 64: 2 x 2 waves of 32 x 32.  BN = 32 (small
// batches: twice the blocks): 2 x 1 waves of 32 x 32, the two wave pairs take alternate
// k-steps and their partial sums meet in LDS at the end.  The next slab is fetched into
// registers (16-byte loads when K allows) while the current one is multiplied, so a block
// pays the memory latency once and not once per slab.
// Result layout of the MFMA: lane -> column lane % 32, register r -> row 8 (r/4) + 4 (lane/32) + r%4.
typedef float v16f __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------------
// Real-valued dense layer with +-1 weights on the bf16 matrix cores.  A float is the exact sum
// of three bf16 values (8 + 8 + 8 significant bits: x = hi + mid + lo, each obtained by
// truncation and an exact subtraction) and a +-1 weight IS a bf16 value, so
//   sum_k x_k w_k = sum_k hi_k w_k + sum_k mid_k w_k + sum_k lo_k w_k
// with every product exact and fp32 accumulation: three bf16 MFMAs (2.5 PFLOP/s) replace one
// fp32 MFMA (157 TFLOP/s).  Weights that are not representable in bf16 would be truncated to 8
// significant bits; the layers of a binary network (Sec. 4.3: real-valued input, binary
// weights) never are.
//   block tile BM x 128, 2 x 2 waves of (BM/2) x 64, K in slabs of 64 (four 32x32x16 steps);
//   the slab is converted on its way from registers to LDS, where it sits row-major in bf16
//   with a row pitch of 144 bytes (16-byte operand reads without bank conflicts).
// ---------------------------------------------------------------------------------
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t pack_hi16(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// the three bf16 terms of four floats, as packed pairs (k, k+1), (k+2, k+3)
__device__ __forceinline__ void split3(const float4 v, uint2 &hi, uint2 &mid, uint2 &lo)
{
    const float x[4] = {v.x, v.y, v.z, v.w};
    uint32_t h[4], m[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        h[i] = __float_as_uint(x[i]) & 0xffff0000u;
        const float r1 = x[i] - __uint_as_float(h[i]);
        m[i] = __float_as_uint(r1) & 0xffff0000u;
        l[i] = __float_as_uint(r1 - __uint_as_float(m[i]));    // at most 8 significant bits are left
    }
    hi = make_uint2(pack_hi16(h[0], h[1]), pack_hi16(h[2], h[3]));
    mid = make_uint2(pack_hi16(m[0], m[1]), pack_hi16(m[2], m[3]));
    lo = make_uint2(pack_hi16(l[0], l[1]), pack_hi16(l[2], l[3]));
}

// WBITS: the weights arrive bit-packed ([N][ceil(K/64)] words as from esp_pack_f32, bit 1 = +1):
// a thread fetches the dword that holds the four bits of its unit and expands them to +-1 bf16
// values on the way to LDS (1/32 of the weight traffic).
template <int BM, int G, bool VEC4, bool FUSE, bool WBITS>
__global__ __launch_bounds__(256)
void dense_bf16x3_kernel(const float *__restrict__ X, const void *__restrict__ Wv, float *__restrict__ Y,
                         const float *__restrict__ thr, const float *__restrict__ sgn,
                         uint64_t *__restrict__ bits, int M, int N, int K)
{
    const float *__restrict__ Wt = static_cast<const float *>(Wv);
    const uint32_t *__restrict__ Wb = static_cast<const uint32_t *>(Wv);
    const int wrow_dw = 2 * ((K + 63) / 64);
    constexpr int BN = 64 * G, BK = 64, PITCH = 72;       // bf16 elements per LDS row (144 bytes)
    constexpr int FM = BM / 64;                           // 32-row blocks per wave
    constexpr int XQ = BM * BK / 4 / 256, WQ = BN * BK / 4 / 256;
    __shared__ __align__(16) uint16_t Xs[3][BM][PITCH];
    __shared__ __align__(16) uint16_t Ws[BN][PITCH];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    // unit u = tid + i * 256 -> row u / 16, k offset 4 * (u % 16): 16 lanes read 256 contiguous
    // bytes; rows beyond the matrix read the last row (their results are not stored), the K tail
    // reads 0
    float4 xr[XQ], wr[WBITS ? 1 : WQ];
    uint32_t wdw[WBITS ? WQ : 1];
    auto fetch = [&](const float *base, int row, int rows, int k0, int u) {
        const int r = min(row + u / 16, rows - 1), k = k0 + 4 * (u % 16);
        const float *p = base + (int64_t)r * K;
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (VEC4) {
            if (k < K)
                v = *reinterpret_cast<const float4 *>(p + k);   // K % 4 == 0: whole or nothing
        } else {
            if (k + 0 < K) v.x = p[k + 0];
            if (k + 1 < K) v.y = p[k + 1];
            if (k + 2 < K) v.z = p[k + 2];
            if (k + 3 < K) v.w = p[k + 3];
        }
        return v;
    };
    auto prefetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < XQ; ++i)
            xr[i] = fetch(X, m0, M, k0, tid + i * 256);
#pragma unroll
        for (int i = 0; i < WQ; ++i) {
            const int u = tid + i * 256;
            if constexpr (WBITS)   // k0 is a multiple of 64 < K, so the dword lies inside the row
                wdw[i] = Wb[(int64_t)min(n0 + u / 16, N - 1) * wrow_dw + (k0 + 4 * (u % 16)) / 32];
            else
                wr[i] = fetch(Wt, n0, N, k0, u);
        }
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < XQ; ++i) {
            const int u = tid + i * 256, r = u / 16, k = 4 * (u % 16);
            uint2 hi, mid, lo;
            split3(xr[i], hi, mid, lo);
            *reinterpret_cast<uint2 *>(&Xs[0][r][k]) = hi;
            *reinterpret_cast<uint2 *>(&Xs[1][r][k]) = mid;
            *reinterpret_cast<uint2 *>(&Xs[2][r][k]) = lo;
        }
#pragma unroll
        for (int i = 0; i < WQ; ++i) {
            const int u = tid + i * 256, r = u / 16, k = 4 * (u % 16);
            if constexpr (WBITS) {
                // bit b -> bf16 +1 (0x3F80) or -1 (0xBF80); beyond K the inputs are 0, so the
                // value there does not matter
                const uint32_t nib = wdw[i] >> (k % 32);
                *reinterpret_cast<uint2 *>(&Ws[r][k]) =
                    make_uint2(0xBF80BF80u ^ ((nib & 1u) << 15) ^ ((nib & 2u) << 30),
                               0xBF80BF80u ^ ((nib & 4u) << 13) ^ ((nib & 8u) << 28));
            } else {
                const float4 w = wr[i];
                *reinterpret_cast<uint2 *>(&Ws[r][k]) =
                    make_uint2(pack_hi16(__float_as_uint(w.x), __float_as_uint(w.y)),
                               pack_hi16(__float_as_uint(w.z), __float_as_uint(w.w)));
            }
        }
    };

    const int lane = tid % kWave, wave = tid / kWave;
    const int lr = lane % 32, half = lane / 32;
    const int wm = (wave % 2) * (BM / 2);    // wave's row offset
    const int wn = (wave / 2) * (32 * G);    // wave's column offset: a 64-column word (G = 2) or half of one
    float th[G], sg[G];                      // FUSE: threshold and sign of the lane's columns
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const int n = n0 + wn + g * 32 + lr;
        th[g] = (FUSE && n < N) ? thr[n] : 0.0f;
        sg[g] = (FUSE && n < N) ? sgn[n] : 1.0f;
    }
    v16f acc[FM][G];
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[f][g][r] = 0.0f;
    prefetch(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
        commit();
        __syncthreads();
        if (k0 + BK < K)
            prefetch(k0 + BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int ko = ks * 16 + 8 * half;
            v8bf b[G];
#pragma unroll
            for (int g = 0; g < G; ++g)
                b[g] = *reinterpret_cast<const v8bf *>(&Ws[wn + g * 32 + lr][ko]);
#pragma unroll
            for (int f = 0; f < FM; ++f)
#pragma unroll
                for (int t = 2; t >= 0; --t) {     // smallest term first
                    const v8bf a = *reinterpret_cast<const v8bf *>(&Xs[t][wm + f * 32 + lr][ko]);
#pragma unroll
                    for (int g = 0; g < G; ++g)
                        acc[f][g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[g], acc[f][g], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    if (!FUSE || Y) {
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int n = n0 + wn + g * 32 + lr;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm + f * 32 + 8 * (r / 4) + 4 * half + r % 4;
                    if (m < M && n < N)
                        Y[(int64_t)m * N + n] = acc[f][g][r];
                }
            }
    }
    if (FUSE) {
        // the comparison masks of a wave's column blocks are 32-bit pieces of the output words:
        // lanes 0 and 32 drop them into a table [row][piece], then one thread per (row, word) stores
        uint32_t *wt = reinterpret_cast<uint32_t *>(&Xs[0][0][0]);     // [BM][2 G], the slabs are done
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
            for (int r = 0; r < 16; ++r)
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const uint64_t mask = __ballot(n0 + wn + g * 32 + lr < N && sg[g] * acc[f][g][r] >= th[g]);
                    const uint32_t piece = half ? (uint32_t)(mask >> 32) : (uint32_t)mask;
                    if (lr == 0)
                        wt[(wm + f * 32 + 8 * (r / 4) + 4 * half + r % 4) * (2 * G) + (wn / 32) + g] = piece;
                }
        __syncthreads();
        const int Nw = (N + 63) / 64;
        for (int t = tid; t < BM * G; t += 256) {
            const int row = m0 + t / G, w = n0 / 64 + t % G;
            if (row < M && w < Nw)
                bits[(int64_t)row * Nw + w] = reinterpret_cast<const uint64_t *>(wt)[t];
        }
    }
}

template <int BN, bool VEC4>
__global__ __launch_bounds__(256)
void dense_f32_mfma_kernel(const float *__restrict__ X, const float *__restrict__ Wt,
                           float *__restrict__ Y, int M, int N, int K)
{
    constexpr int BM = 64, BK = 32;
    constexpr int XQ = BM * BK / 4 / 256;   // float4 units per thread and slab: 2
    constexpr int WQ = BN * BK / 4 / 256;   // 2 (BN = 64) or 1 (BN = 32)
    __shared__ float Xs[BK][BM + 4];
    __shared__ float Ws[BK][BN + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    // unit u = tid + i * 256 -> row u / 8, k offset 4 * (u % 8): 8 lanes read 128 contiguous bytes
    float4 xr[XQ], wr[WQ];
    auto fetch = [&](const float *base, int row, int rows, int k0, int u) {
        const int r = row + u / 8, k = k0 + 4 * (u % 8);
        float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (r < rows) {
            const float *p = base + (int64_t)r * K + k;
            if (VEC4) {
                if (k < K)
                    v = *reinterpret_cast<const float4 *>(p);   // K % 4 == 0: whole or nothing
            } else {
                if (k + 0 < K) v.x = p[0];
                if (k + 1 < K) v.y = p[1];
                if (k + 2 < K) v.z = p[2];
                if (k + 3 < K) v.w = p[3];
            }
        }
        return v;
    };
    auto prefetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < XQ; ++i)
            xr[i] = fetch(X, m0, M, k0, tid + i * 256);
#pragma unroll
        for (int i = 0; i < WQ; ++i)
            wr[i] = fetch(Wt, n0, N, k0, tid + i * 256);
    };
    auto commit = [&]() {
#pragma unroll
        for (int i = 0; i < XQ; ++i) {
            const int u = tid + i * 256, r = u / 8, k = 4 * (u % 8);
            Xs[k + 0][r] = xr[i].x;
            Xs[k + 1][r] = xr[i].y;
            Xs[k + 2][r] = xr[i].z;
            Xs[k + 3][r] = xr[i].w;
        }
#pragma unroll
        for (int i = 0; i < WQ; ++i) {
            const int u = tid + i * 256, r = u / 8, k = 4 * (u % 8);
            Ws[k + 0][r] = wr[i].x;
            Ws[k + 1][r] = wr[i].y;
            Ws[k + 2][r] = wr[i].z;
            Ws[k + 3][r] = wr[i].w;
        }
    };

    const int lane = tid % kWave, wave = tid / kWave;
    const int lr = lane % 32, half = lane / 32;
    constexpr int WN = BN / 32;              // waves along N: 2 or 1
    const int wm = (wave % 2) * 32;          // wave's row offset
    const int wn = WN == 2 ? (wave / 2) * 32 : 0;
    const int kpart = WN == 2 ? 0 : wave / 2;   // BN = 32: which of the alternate k-steps
    v16f acc;
#pragma unroll
    for (int r = 0; r < 16; ++r)
        acc[r] = 0.0f;
    prefetch(0);
    for (int k0 = 0; k0 < K; k0 += BK) {
        commit();
        __syncthreads();
        if (k0 + BK < K)
            prefetch(k0 + BK);
#pragma unroll
        for (int st = 0; st < BK / 2 / (3 - WN); ++st) {
            const int k = 2 * (WN == 2 ? st : 2 * st + kpart) + half;
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(Xs[k][wm + lr], Ws[k][wn + lr], acc, 0, 0, 0);
        }
        __syncthreads();
    }
    bool owner = true;                       // this wave holds finished sums
    if (WN == 1) {
        // the wave pairs 0,1 and 2,3 hold partial sums of the same 64 x 32 tile
        float *red = &Xs[0][0];              // 32 x 68 floats >= 2 waves x 16 x 64
        owner = wave < 2;
        if (!owner) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                red[((wave - 2) * 16 + r) * kWave + lane] = acc[r];
        }
        __syncthreads();
        if (owner) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[r] += red[(wave * 16 + r) * kWave + lane];
        }
    }
    const int n = n0 + wn + lr;
    if (owner) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + wm + 8 * (r / 4) + 4 * half + r % 4;
            if (m < M && n < N)
                Y[(int64_t)m * N + n] = acc[r];
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

// Small batch with the folded batch-norm threshold + sign in the epilogue (the network of
// Sec. 6.2 evaluated one image at a time): a block of WAVES waves owns 4 * WAVES = 64 or 16
// consecutive neurons, i.e. one packed output word, or one 16-bit quarter of it, per row of
// X (16 when 64 would leave most CUs without a block); every wave streams the weight rows
// of 4 neurons (all four in flight together), the lanes stride over K, a butterfly sums.
// bit n of row m = (sgn[n] * y[m][n] >= thr[n]); pre (if not null) also receives y.
template <int MS, bool VEC4, int WAVES>
__global__ __launch_bounds__(WAVES * 64)
void dense_f32_gemv_bits_kernel(const float *__restrict__ X, const float *__restrict__ Wt,
                                const float *__restrict__ thr, const float *__restrict__ sgn,
                                uint64_t *__restrict__ bits, float *__restrict__ pre, int M, int N, int K)
{
    constexpr int NPW = 4;                       // neurons per wave
    constexpr int RB = NPW * WAVES;              // neurons per block: 64 or 16
    __shared__ unsigned char decided[MS][RB];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int n_blk = blockIdx.x * RB;
    const int nl0 = wave * NPW;
    float acc[NPW][MS];
#pragma unroll
    for (int j = 0; j < NPW; ++j)
#pragma unroll
        for (int m = 0; m < MS; ++m)
            acc[j][m] = 0.0f;
    // rows beyond N read the last row: their results are never used
    const float *wrow[NPW];
#pragma unroll
    for (int j = 0; j < NPW; ++j)
        wrow[j] = Wt + (int64_t)min(n_blk + nl0 + j, N - 1) * K;
    if (VEC4) {
        for (int k = 4 * lane; k < K; k += 4 * kWave) {
            float4 w[NPW];
#pragma unroll
            for (int j = 0; j < NPW; ++j)
                w[j] = *reinterpret_cast<const float4 *>(wrow[j] + k);
#pragma unroll
            for (int m = 0; m < MS; ++m) {
                if (m >= M)
                    continue;
                const float4 x = *reinterpret_cast<const float4 *>(X + (int64_t)m * K + k);
#pragma unroll
                for (int j = 0; j < NPW; ++j) {
                    acc[j][m] = fmaf(x.x, w[j].x, acc[j][m]);
                    acc[j][m] = fmaf(x.y, w[j].y, acc[j][m]);
                    acc[j][m] = fmaf(x.z, w[j].z, acc[j][m]);
                    acc[j][m] = fmaf(x.w, w[j].w, acc[j][m]);
                }
            }
        }
    } else {
        for (int k = lane; k < K; k += kWave) {
            float w[NPW];
#pragma unroll
            for (int j = 0; j < NPW; ++j)
                w[j] = wrow[j][k];
#pragma unroll
            for (int m = 0; m < MS; ++m) {
                if (m >= M)
                    continue;
                const float x = X[(int64_t)m * K + k];
#pragma unroll
                for (int j = 0; j < NPW; ++j)
                    acc[j][m] = fmaf(x, w[j], acc[j][m]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NPW; ++j) {
        const int n = n_blk + nl0 + j;
        const int nc = min(n, N - 1);
        const float t = thr[nc], sg = sgn[nc];
#pragma unroll
        for (int m = 0; m < MS; ++m) {
            float v = acc[j][m];
            for (int off = 32; off > 0; off >>= 1)
                v += __shfl_xor(v, off, kWave);
            if (lane == 0) {
                decided[m][nl0 + j] = n < N && sg * v >= t;
                if (pre && n < N && m < M)
                    pre[(int64_t)m * N + n] = v;
            }
        }
    }
    __syncthreads();
    for (int m = wave; m < M; m += WAVES) {
        const uint64_t word = __ballot(lane < RB && decided[m][lane % RB] != 0);
        if (lane != 0)
            continue;
        if (RB == 64)
            bits[(int64_t)m * gridDim.x + blockIdx.x] = word;
        else   // 16-bit piece blockIdx.x % 4 of word blockIdx.x / 4 (little-endian)
            reinterpret_cast<uint16_t *>(bits)[(int64_t)m * gridDim.x + blockIdx.x] = (uint16_t)word;
    }
}

// The same layer for up to 4 input rows with the weights bit-packed ([N][ceil(K/64)] words as
// from esp_pack_f32, bit 1 = +1): a lane takes 8 consecutive k per step, i.e. one byte of each
// of its wave's 4 weight rows and 8 inputs per row of X, and adds or subtracts each input
// (x XOR sign bit, then add).  1/32 of the weight traffic of the float form, which is what a
// network evaluated one image at a time spends its first layer on.
template <int MS, bool VEC8, int WAVES>
__global__ __launch_bounds__(WAVES * 64)
void dense_f32_bw_gemv_bits_kernel(const float *__restrict__ X, const uint32_t *__restrict__ Wb,
                                   const float *__restrict__ thr, const float *__restrict__ sgn,
                                   uint64_t *__restrict__ bits, float *__restrict__ pre, int M, int N, int K)
{
    constexpr int NPW = 4;                       // neurons per wave
    constexpr int RB = NPW * WAVES;              // neurons per block: 64 or 16
    __shared__ unsigned char decided[MS][RB];
    const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
    const int n_blk = blockIdx.x * RB;
    const int nl0 = wave * NPW;
    const int row_dw = 2 * ((K + 63) / 64);
    float acc[NPW][MS];
#pragma unroll
    for (int j = 0; j < NPW; ++j)
#pragma unroll
        for (int m = 0; m < MS; ++m)
            acc[j][m] = 0.0f;
    // rows beyond N read the last row: their results are never used
    const uint32_t *wrow[NPW];
#pragma unroll
    for (int j = 0; j < NPW; ++j)
        wrow[j] = Wb + (int64_t)min(n_blk + nl0 + j, N - 1) * row_dw;
    for (int k = 8 * lane; k < K; k += 8 * kWave) {
        uint32_t wbyte[NPW];
#pragma unroll
        for (int j = 0; j < NPW; ++j)
            wbyte[j] = wrow[j][k / 32] >> (k % 32);      // bits k .. k+7 in the low byte
#pragma unroll
        for (int m = 0; m < MS; ++m) {
            if (m >= M)
                continue;
            const float *xp = X + (int64_t)m * K + k;
            float x[8];
            if (VEC8) {                                   // K % 8 == 0: whole steps, 16-byte loads
                const float4 lo = *reinterpret_cast<const float4 *>(xp);
                const float4 hi = *reinterpret_cast<const float4 *>(xp + 4);
                x[0] = lo.x, x[1] = lo.y, x[2] = lo.z, x[3] = lo.w;
                x[4] = hi.x, x[5] = hi.y, x[6] = hi.z, x[7] = hi.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    x[e] = k + e < K ? xp[e] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < NPW; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    // bit 1: + x, bit 0: - x
                    const uint32_t flipsign = (~(wbyte[j] >> e) & 1u) << 31;
                    acc[j][m] += __uint_as_float(__float_as_uint(x[e]) ^ flipsign);
                }
        }
    }
#pragma unroll
    for (int j = 0; j < NPW; ++j) {
        const int n = n_blk + nl0 + j;
        const int nc = min(n, N - 1);
        const float t = thr[nc], sg = sgn[nc];
#pragma unroll
        for (int m = 0; m < MS; ++m) {
            float v = acc[j][m];
            for (int off = 32; off > 0; off >>= 1)
                v += __shfl_xor(v, off, kWave);
            if (lane == 0) {
                decided[m][nl0 + j] = n < N && sg * v >= t;
                if (pre && n < N && m < M)
                    pre[(int64_t)m * N + n] = v;
            }
        }
    }
    __syncthreads();
    for (int m = wave; m < M; m += WAVES) {
        const uint64_t word = __ballot(lane < RB && decided[m][lane % RB] != 0);
        if (lane != 0)
            continue;
        if (RB == 64)
            bits[(int64_t)m * gridDim.x + blockIdx.x] = word;
        else   // 16-bit piece blockIdx.x % 4 of word blockIdx.x / 4 (little-endian)
            reinterpret_cast<uint16_t *>(bits)[(int64_t)m * gridDim.x + blockIdx.x] = (uint16_t)word;
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

// Fast path for the 3x3x3 first layer of the Sec. 6.3 network at stride 1, on the bf16 matrix
// cores: every window value is split exactly into three bf16 terms (split3) and the +-1 filter
// values are bf16 values, so three v_mfma_f32_32x32x16_bf16 per k-step give the fp32 sum of
// exact products (a filter value that is not representable in bf16 would be cut to 8
// significant bits).  The layer is the dense contraction
//   out[pixel][l2] = sum_k window[pixel][k] * filt[l2][k],  k = (dy, dx, c) < 27 (padded to 32),
// so a wave owns a strip of 32 consecutive output pixels of one output row (= the 32 rows of
// the MFMA's A operand) and NB blocks of 32 output channels (the columns):
//  * the wave copies the strip's input window (3 rows x 34 pixels x 3 channels, zeros outside
//    the image) into its private LDS slice; lane (pixel p, k-half h) reads the elements
//    (p, k = 16 s + 8 h + j), j = 0..7, of the lowered window for step s straight from there;
//  * the weights of the wave's channels stay in registers as B operands for all its strips;
//  * with FUSE the per-channel sign of the folded batch-norm is multiplied into the weights
//    (exact), so the epilogue is one compare per accumulator whose 64-lane mask holds the
//    bits of two pixels x 32 channels; only packed words leave the kernel (the pre-
//    activations are written as well only if `pre` is given).
// MFMA result layout: lane -> column lane % 32, register r -> row 8 (r / 4) + 4 (lane / 32) + r % 4.

// v or +0.0f.  A bit mask instead of a select keeps the load that produced v unconditional
// (from a clamped, always valid address), so that independent loads are issued back to back
// rather than each inside its own branch with its own wait.
__device__ __forceinline__ float keep_if(float v, bool keep)
{
    return __uint_as_float(__float_as_uint(v) & (keep ? 0xffffffffu : 0u));
}

template <int NB, bool FUSE>
__global__ __launch_bounds__(256, 2)
void conv3x3x3_mfma_kernel(const float *__restrict__ in, const float *__restrict__ filt,
                           float *__restrict__ pre, const float *__restrict__ thr,
                           const float *__restrict__ sgn, uint64_t *__restrict__ bits,
                           int H, int W, int L2, int pad, int H2, int W2, int strips, int rows_strips,
                           int tasks)
{
    constexpr int T = 27, KS = 2;                  // taps * channels, k-steps of 16 (k padded to 32)
    constexpr int PIX = 32, WROW = (PIX + 2) * 3;  // floats per window row
    constexpr int WIN = 3 * WROW;
    static_assert(NB == 1 || NB == 4, "one block per wave (32-bit output pieces) or whole words");
    __shared__ float win_all[4][WIN + 2];          // + a zero slot for the padding k = 27, + scratch
    __shared__ __align__(16) uint32_t word_all[4][PIX * NB];   // [pixel][block] mask halves
    __shared__ float filt_s[NB * 32 * T];          // the filters of one channel group, [channel][k]

    const int lane = threadIdx.x % kWave;
    // the wave index and everything derived from it (the task decomposition) stay in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int lr = lane % 32, half = lane / 32;
    float *win = win_all[wave];
    if (lane == 0)
        win[WIN] = 0.0f;

    // The filters of the channel group of the block's first task travel through LDS: read
    // per lane they are a gather with a stride of 27 floats (32 cache lines per load).  A wave
    // that later moves on to another group gathers them directly.
    const int cg_staged = (blockIdx.x * (blockDim.x / kWave)) / rows_strips;
    {
        const int64_t base = (int64_t)cg_staged * NB * 32 * T;
        for (int i = threadIdx.x; i < NB * 32 * T; i += blockDim.x)
            filt_s[i] = base + i < (int64_t)L2 * T ? filt[base + i] : 0.0f;
        __syncthreads();
    }

    // window element i = lane + 64 q of a strip: row wr, pixel wx, offset wo from the window's
    // first element in the image (i beyond the window: a row that is never inside the image)
    constexpr int kTrips = (WIN + kWave - 1) / kWave;
    int wr[kTrips], wx[kTrips], wo[kTrips], wdst[kTrips];
#pragma unroll
    for (int q = 0; q < kTrips; ++q) {
        const int i = lane + q * kWave;
        const int r = i / WROW, j = i - r * WROW;
        wr[q] = i < WIN ? r : -(1 << 30);
        wx[q] = j / 3;
        wo[q] = r * W * 3 + j;
        wdst[q] = i < WIN ? i : WIN + 1;           // WIN + 1: scratch slot
    }

    // lowered-window element (pixel lr, k) sits at 93 * dy + 3 * lr + k, dy = k / 9; a lane's
    // operand of k-step s holds k = 16 s + 8 half + j, j = 0..7 (k >= 27: the zero slot)
    int off[KS][8];
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int k = 16 * s + 8 * half + j;
            off[s][j] = k < T ? 93 * (k / 9) + 3 * lr + k : WIN;
        }

    const int Cw = (L2 + 63) / 64;
    v8bf bw[NB][KS];       // filter values x folded sign: +-1 (or 0), exact in bf16
    float th[NB], sg[NB];
    int cur_cg = -1;
    const int nwaves = gridDim.x * (blockDim.x / kWave);
    const int task0 = blockIdx.x * (blockDim.x / kWave) + wave;

    // The window of a strip is fetched one task ahead: its loads are in flight while the
    // matrix cores work on the current strip.  Zero padding is applied here; window rows are
    // contiguous runs of the image; 32-bit offsets from the image's first element
    // (H * W * 3 < 2^31, checked by the host).
    float wv_[kTrips];
    bool winb_[kTrips];    // inside the image; applied when the value moves to LDS, so that
                           // nothing waits for the loads where they are issued
    auto fetch_window = [&](int task) {
        const int rs = task % rows_strips;
        const int bm = rs / strips;
        const int n0 = (rs - bm * strips) * PIX;
        const float *img = in + (int64_t)(bm / H2) * H * W * 3;
        const int y0 = bm % H2 - pad, x0 = n0 - pad;
        const int first = (y0 * W + x0) * 3;
#pragma unroll
        for (int q = 0; q < kTrips; ++q) {
            const bool inb = (unsigned)(y0 + wr[q]) < (unsigned)H && (unsigned)(x0 + wx[q]) < (unsigned)W;
            wv_[q] = img[inb ? first + wo[q] : 0];
            winb_[q] = inb;
        }
    };
    if (task0 < tasks)
        fetch_window(task0);

    for (int task = task0; task < tasks; task += nwaves) {
        // task -> (channel group, image row bm = b * H2 + m, strip); channel group slowest
        const int cg = task / rows_strips;
        const int rs = task - cg * rows_strips;
        const int bm = rs / strips;
        const int n0 = (rs - bm * strips) * PIX;
        if (cg != cur_cg) {     // wave-uniform
            cur_cg = cg;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int l2 = (cg * NB + nb) * 32 + lr;
                const bool ok = l2 < L2;
                const int l2c = ok ? l2 : 0;          // loads stay unconditional (and in flight together)
                sg[nb] = FUSE ? sgn[l2c] : 1.0f;
                th[nb] = FUSE ? thr[l2c] : 0.0f;
                if (!ok) {
                    sg[nb] = 1.0f;
                    th[nb] = __builtin_inff();         // beyond L2: bit 0
                }
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    float wv[8];
                    if (cg == cg_staged) {            // wave-uniform
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            wv[j] = filt_s[(nb * 32 + lr) * T + min(16 * s + 8 * half + j, T - 1)];
                    } else {
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            wv[j] = filt[(int64_t)l2c * T + min(16 * s + 8 * half + j, T - 1)];
                    }
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        bw[nb][s][j] = (__bf16)keep_if(sg[nb] * wv[j], ok && 16 * s + 8 * half + j < T);
                }
            }
        }

        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int q = 0; q < kTrips; ++q)
            win[wdst[q]] = keep_if(wv_[q], winb_[q]);
        __builtin_amdgcn_wave_barrier();   // LDS operations of one wave complete in order
        if (task + nwaves < tasks)
            fetch_window(task + nwaves);

        v16f acc[NB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[nb][r] = 0.0f;
        // every window value is the exact sum of three bf16 terms (see split3) and the weights
        // are +-1, so three bf16 MFMAs per k-step give the fp32 sum of exact products
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            uint2 hi[2], mid[2], lo[2];
#pragma unroll
            for (int q = 0; q < 2; ++q)
                split3(make_float4(win[off[s][4 * q]], win[off[s][4 * q + 1]], win[off[s][4 * q + 2]],
                                   win[off[s][4 * q + 3]]), hi[q], mid[q], lo[q]);
            const uint4 a3[3] = {make_uint4(lo[0].x, lo[0].y, lo[1].x, lo[1].y),
                                 make_uint4(mid[0].x, mid[0].y, mid[1].x, mid[1].y),
                                 make_uint4(hi[0].x, hi[0].y, hi[1].x, hi[1].y)};
#pragma unroll
            for (int t = 0; t < 3; ++t) {
                v8bf a;
                __builtin_memcpy(&a, &a3[t], 16);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bw[nb][s], acc[nb], 0, 0, 0);
            }
        }

        const int64_t pix0 = (int64_t)bm * W2 + n0;    // first output pixel of the strip
        if (!FUSE || pre) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int l2 = (cg * NB + nb) * 32 + lr;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int p = 8 * (r / 4) + 4 * half + r % 4;
                    if (l2 < L2 && n0 + p < W2)
                        pre[(pix0 + p) * L2 + l2] = sg[nb] * acc[nb][r];   // sg = +-1: undoes the fold
                }
            }
        }
        if (FUSE) {
            // comparison mask of register r, block nb: low half = the 32 channel bits of pixel
            // 8 (r/4) + r%4, high half = those of that pixel + 4.  Lanes 0 and 32 drop the halves
            // into the wave's LDS word table [pixel][block]; lane p then stores pixel p's words.
            if constexpr (NB == 1) {
                // one 32-channel block per wave (small grids): the mask halves are 32-bit pieces
                // of the output words, stored straight from lanes 0 and 32
                uint32_t *bits32 = reinterpret_cast<uint32_t *>(bits);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint64_t mask = __ballot(acc[0][r] >= th[0]);
                    const uint32_t v = half ? (uint32_t)(mask >> 32) : (uint32_t)mask;
                    const int p = 8 * (r / 4) + 4 * half + r % 4;
                    if (lr == 0 && n0 + p < W2)
                        bits32[(pix0 + p) * (2 * Cw) + cg] = v;
                }
            } else {
                uint32_t *wl = word_all[wave];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    uint32_t v[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const uint64_t mask = __ballot(acc[nb][r] >= th[nb]);
                        v[nb] = half ? (uint32_t)(mask >> 32) : (uint32_t)mask;
                    }
                    const int p = 8 * (r / 4) + 4 * half + r % 4;
                    if (lr == 0) {
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            wl[p * NB + nb] = v[nb];
                    }
                }
                __builtin_amdgcn_wave_barrier();
                if (lane < PIX && n0 + lane < W2) {
#pragma unroll
                    for (int q = 0; q < NB / 2; ++q) {
                        const int w = cg * (NB / 2) + q;
                        const uint64_t lo = wl[lane * NB + 2 * q];
                        const uint64_t hi = wl[lane * NB + 2 * q + 1];
                        if (w < Cw)
                            bits[(pix0 + lane) * Cw + w] = lo | (hi << 32);
                    }
                }
            }
        }
    }
}

} // namespace esp

namespace esp {

// Tiled float dense layer: with bits != null the fused layer on the bf16 matrix cores (threshold
// epilogue, Y optional), else the plain fp32 product.
static int dense_mfma_launch(const float *X, const float *W, float *Y, const float *thr, const float *sgn,
                             uint64_t *bits, int64_t M, int64_t N, int64_t K, hipStream_t s,
                             const uint64_t *Wbits = nullptr)
{
    const int64_t gy = ceil_div(M, 64);
    if (gy > 65535)
        return ESP_ESHAPE;
    const bool vec4 = K % 4 == 0 && aligned(X, 16) && (Wbits || aligned(W, 16));
    if (bits) {
        // the fused layer of a binary network (+-1 weights): the bf16 matrix cores, three exact
        // terms per input.  Measured on the MLP's first layer (N = 4096, K = 784) at 8 ... 256 /
        // 512 / 1024 rows: 15.6 / 19.0 / 25.9 us (the fp32 kernel below: 17.4 ... 26 / 38 / 67 us)
        // 128 x 128 tiles when there are many of them, else 64 x 128, else 64 x 64: the kernel is
        // bound by the chain of its K slabs, so it wants several blocks per CU
        const int64_t t128 = ceil_div(M, 128) * ceil_div(N, 128);
        const int bm = t128 >= 1024 ? 128 : 64;
        const int g = (bm == 128 || ceil_div(M, 64) * ceil_div(N, 128) >= 512) ? 2 : 1;
        const dim3 grid((unsigned)ceil_div(N, 64 * g), (unsigned)ceil_div(M, bm));
#define ESP_DENSE_BF16(BMV, GV, V)                                                                         \
    do {                                                                                                   \
        if (Wbits)                                                                                         \
            hipLaunchKernelGGL((dense_bf16x3_kernel<BMV, GV, V, true, true>), grid, dim3(256), 0, s, X,    \
                               static_cast<const void *>(Wbits), Y, thr, sgn, bits, (int)M, (int)N, (int)K); \
        else                                                                                               \
            hipLaunchKernelGGL((dense_bf16x3_kernel<BMV, GV, V, true, false>), grid, dim3(256), 0, s, X,   \
                               static_cast<const void *>(W), Y, thr, sgn, bits, (int)M, (int)N, (int)K);   \
    } while (0)
        if (bm == 128 && vec4)
            ESP_DENSE_BF16(128, 2, true);
        else if (bm == 128)
            ESP_DENSE_BF16(128, 2, false);
        else if (g == 2 && vec4)
            ESP_DENSE_BF16(64, 2, true);
        else if (g == 2)
            ESP_DENSE_BF16(64, 2, false);
        else if (vec4)
            ESP_DENSE_BF16(64, 1, true);
        else
            ESP_DENSE_BF16(64, 1, false);
#undef ESP_DENSE_BF16
        return launch_status();
    }
    const bool narrow = gy * ceil_div(N, 64) < 256;   // few blocks: halve the tile width
    const dim3 grid((unsigned)ceil_div(N, narrow ? 32 : 64), (unsigned)gy);
#define ESP_DENSE(BN, V)                                                                                   \
    hipLaunchKernelGGL((dense_f32_mfma_kernel<BN, V>), grid, dim3(256), 0, s, X, W, Y, (int)M, (int)N, (int)K)
    if (narrow && vec4)
        ESP_DENSE(32, true);
    else if (narrow)
        ESP_DENSE(32, false);
    else if (vec4)
        ESP_DENSE(64, true);
    else
        ESP_DENSE(64, false);
#undef ESP_DENSE
    return launch_status();
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
    return dense_mfma_launch(X, W, Y, nullptr, nullptr, nullptr, M, N, K, s);
}

extern "C" int esp_dense_f32_bn_sign_pack(const float *X, const float *W, const float *thr, const float *sgn,
                                          uint64_t *bits, float *pre, int64_t M, int64_t N, int64_t K,
                                          esp_stream stream)
{
    using namespace esp;
    if (M < 0 || N <= 0 || K <= 0)
        return ESP_EINVAL;
    if (M >= (1ll << 31) || N >= (1ll << 31) || K >= (1ll << 31))
        return ESP_ESHAPE;
    if (M == 0)
        return ESP_OK;
    if (!X || !W || !thr || !sgn || !bits)
        return ESP_EINVAL;
    if (!aligned(X, 4) || !aligned(W, 4) || !aligned(thr, 4) || !aligned(sgn, 4) || !aligned(bits, 8) ||
        (pre && !aligned(pre, 4)))
        return ESP_EALIGN;
    if (M > 4)   // larger batches: the matrix-core kernel with the threshold epilogue
        return dense_mfma_launch(X, W, pre, thr, sgn, bits, M, N, K, as_stream(stream));
    const bool vec4 = K % 4 == 0 && aligned(X, 16) && aligned(W, 16);
    // 64 neurons per block when that gives every CU a block, else 16; the grid covers every
    // 16-bit piece of the output words, also those beyond N (zeros)
    const int64_t Nw = ceil_div(N, 64);
    const bool wide = Nw >= 256;
    const dim3 grid((unsigned)(wide ? Nw : 4 * Nw));
    hipStream_t s = as_stream(stream);
#define ESP_GEMV_BITS_F32(MS, V)                                                                           \
    do {                                                                                                   \
        if (wide)                                                                                          \
            hipLaunchKernelGGL((dense_f32_gemv_bits_kernel<MS, V, 16>), grid, dim3(1024), 0, s, X, W, thr, \
                               sgn, bits, pre, (int)M, (int)N, (int)K);                                    \
        else                                                                                               \
            hipLaunchKernelGGL((dense_f32_gemv_bits_kernel<MS, V, 4>), grid, dim3(256), 0, s, X, W, thr,   \
                               sgn, bits, pre, (int)M, (int)N, (int)K);                                    \
    } while (0)
    if (M == 1 && vec4)
        ESP_GEMV_BITS_F32(1, true);
    else if (M == 1)
        ESP_GEMV_BITS_F32(1, false);
    else if (vec4)
        ESP_GEMV_BITS_F32(4, true);
    else
        ESP_GEMV_BITS_F32(4, false);
#undef ESP_GEMV_BITS_F32
    return launch_status();
}

extern "C" int esp_dense_f32_bw_bn_sign_pack(const float *X, const uint64_t *Wbits, const float *thr,
                                             const float *sgn, uint64_t *bits, float *pre, int64_t M,
                                             int64_t N, int64_t K, esp_stream stream)
{
    using namespace esp;
    if (M < 0 || N <= 0 || K <= 0)
        return ESP_EINVAL;
    if (M >= (1ll << 31) || N >= (1ll << 31) || K >= (1ll << 30))
        return ESP_ESHAPE;
    if (M == 0)
        return ESP_OK;
    if (!X || !Wbits || !thr || !sgn || !bits)
        return ESP_EINVAL;
    if (!aligned(X, 4) || !aligned(Wbits, 8) || !aligned(thr, 4) || !aligned(sgn, 4) || !aligned(bits, 8) ||
        (pre && !aligned(pre, 4)))
        return ESP_EALIGN;
    hipStream_t s = as_stream(stream);
    if (M > 4)
        return dense_mfma_launch(X, nullptr, pre, thr, sgn, bits, M, N, K, s, Wbits);
    const bool vec8 = K % 8 == 0 && aligned(X, 16);
    const int64_t Nw = ceil_div(N, 64);
    const bool wide = Nw >= 256;
    const dim3 grid((unsigned)(wide ? Nw : 4 * Nw));
    const uint32_t *wb = reinterpret_cast<const uint32_t *>(Wbits);
#define ESP_GEMV_BITS_BW(MS, V)                                                                            \
    do {                                                                                                   \
        if (wide)                                                                                          \
            hipLaunchKernelGGL((dense_f32_bw_gemv_bits_kernel<MS, V, 16>), grid, dim3(1024), 0, s, X, wb,  \
                               thr, sgn, bits, pre, (int)M, (int)N, (int)K);                               \
        else                                                                                               \
            hipLaunchKernelGGL((dense_f32_bw_gemv_bits_kernel<MS, V, 4>), grid, dim3(256), 0, s, X, wb,    \
                               thr, sgn, bits, pre, (int)M, (int)N, (int)K);                               \
    } while (0)
    if (M == 1 && vec8)
        ESP_GEMV_BITS_BW(1, true);
    else if (M == 1)
        ESP_GEMV_BITS_BW(1, false);
    else if (vec8)
        ESP_GEMV_BITS_BW(4, true);
    else
        ESP_GEMV_BITS_BW(4, false);
#undef ESP_GEMV_BITS_BW
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
    // a wave takes 128 output channels (4 MFMA column blocks, whole output words), or, when
    // that leaves most SIMDs without a wave (small batches), 32 channels = a 32-bit piece of a
    // word; either way the groups cover every word completely (channels beyond L2 give 0 bits)
    const int strips = (W2 + 31) / 32;
    const int64_t rows_strips = (int64_t)B * H2 * strips;
    const int64_t Cw = ceil_div(L2, 64);
    const int nb = rows_strips * ceil_div(L2, 128) < 1024 ? 1 : 4;
    const int64_t cgroups = nb == 1 ? 2 * Cw : ceil_div(L2, 128);
    const int64_t tasks = rows_strips * cgroups;
    if (tasks >= (1ll << 31))
        return ESP_OK;
    *done = true;
    // two waves per SIMD stay resident and walk the tasks, so the weights are fetched once per wave
    const int64_t waves = tasks < 2048 ? tasks : 2048;
    const dim3 grid((unsigned)ceil_div(waves, 4));
#define ESP_CONV1(NB, FUSE)                                                                            \
    hipLaunchKernelGGL((conv3x3x3_mfma_kernel<NB, FUSE>), grid, dim3(256), 0, stream, in, filt, out, thr, \
                       sgn, bits, H, W, L2, pad, H2, W2, strips, (int)rows_strips, (int)tasks)
    if (bits) {
        if (nb == 1)
            ESP_CONV1(1, true);
        else
            ESP_CONV1(4, true);
    } else {
        if (nb == 1)
            ESP_CONV1(1, false);
        else
            ESP_CONV1(4, false);
    }
#undef ESP_CONV1
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
