// Binary matrix product on the matrix cores (measured alternative to the XOR-popcount
// kernel for the dense contraction of Sec. 4.2, Eq. 2 of arXiv 1705.07175).
//
// gfx950's block-scaled MFMA takes 4-bit floating-point (E2M1) operands at twice the rate of
// 8-bit ones.  A packed bit needs no real conversion to become such an operand: masking a
// source dword with 0x11111111 << j leaves, in every nibble, either 0 or the E2M1 pattern
// 1, 2 or 4 = 0.5, 1.0 or 2.0, and the instruction's per-block scale (2^1, 2^0, 2^-1) turns
// each of them into exactly 1.  That is one AND per operand dword (bit 3 of a nibble is the
// sign bit, so j = 3 takes a shift first).  Any permutation of k is allowed as long as both
// operands use the same one, so the four masks j = 0..3 of one source dword simply feed
// four successive MFMA calls.
// With a, b in {0,1} the accumulator holds c = sum_k a_k b_k exactly (fp32, c <= K < 2^24),
// and the +-1 dot product follows from the row popcounts:
//   dot = K - 2 * (pa + pb - 2 c) = K - 2 pa - 2 pb + 4 c.
// A 0 bit is -1 throughout, which is also the -1 border of a convolution.  pa and pb are
// counted once per block by the threads that fetch the packed rows from global memory.
//
// Tile: 256 threads = 2 x 2 waves, each wave FM x FN MFMA blocks of 32 x 32
// (v_mfma_scale_f32_32x32x64_f8f6f4): 128 x 64 per wave (two blocks per CU), or 64 x 64 per
// wave (three blocks per CU) for products with fewer than 512 of the large tiles.  Operands
// come from two LDS buffers of packed rows in the same 16-byte k-group layout as the
// XOR-popcount kernel: stage s + 1 is written while stage s is read, one barrier per stage.
// Measured on an 8192-cube: 128 x 128 per wave (accumulators in AGPRs, one wave per SIMD,
// half the ANDs per MFMA) ran 15 % slower than 128 x 64, so it is not instantiated; with
// the operand ANDs, the popcounts and the epilogue all removed the time did not change, the
// loads of a stage (global -> registers -> LDS) and the barrier are what the MFMAs wait for.
#include <type_traits>

#include "esp_internal.h"
#include "tile_sources.h"

namespace esp {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kMfmaKG = 4;                     // 16-byte k-groups per LDS stage (512 bits of K)
constexpr int kMaxMfmaK = 1 << 24;             // fp32 accumulation stays exact

// E8M0 scale bytes: 2^(s - 127)
constexpr int kScale2 = 128, kScale1 = 127, kScaleHalf = 126;

template <int J>
__device__ __forceinline__ v8i encode(const uint4 x)
{
    v8i r;
    if (J < 3) {
        const uint32_t m = 0x11111111u << J;
        r[0] = (int)(x.x & m);
        r[1] = (int)(x.y & m);
        r[2] = (int)(x.z & m);
        r[3] = (int)(x.w & m);
    } else {
        r[0] = (int)((x.x >> 1) & 0x44444444u);
        r[1] = (int)((x.y >> 1) & 0x44444444u);
        r[2] = (int)((x.z >> 1) & 0x44444444u);
        r[3] = (int)((x.w >> 1) & 0x44444444u);
    }
    r[4] = r[5] = r[6] = r[7] = 0;   // unused by 4-bit operands
    return r;
}

template <int J, int FM, int FN>
__device__ __forceinline__ void mfma_group(const uint4 (&xa)[FM], const uint4 (&xb)[FN], v16f (&acc)[FM][FN])
{
    constexpr int sc = J == 0 ? kScale2 : (J == 1 ? kScale1 : kScaleHalf);
    v8i b[FN];
#pragma unroll
    for (int g = 0; g < FN; ++g)
        b[g] = encode<J>(xb[g]);
#pragma unroll
    for (int f = 0; f < FM; ++f) {
        const v8i a = encode<J>(xa[f]);
#pragma unroll
        for (int g = 0; g < FN; ++g)
            acc[f][g] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b[g], acc[f][g], 4, 4, 0, sc, 0, sc);
    }
}

__device__ __forceinline__ int popc4(const uint4 v)
{
    return __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w);
}

struct MfmaOut {
    int32_t *C;             // int32 dots [M][N], or
    uint64_t *bits;         // packed signs [M][Nw]
    const int32_t *thr;
    const uint64_t *flip;
    int Nw;
    int pool_log2w;         // 0: no pooling; else bits is [M/4][Nw] behind a fused 2x2 max-pool
                            // and this is log2 of the convolution's output width W2
    int vec_store;          // C is 16-byte aligned and N a multiple of 4: 16-byte stores
    const int32_t *wsum;    // bit-plane mode (Eq. 3): rows 8j .. 8j+7 of A are the planes of input
                            // row j; C (optional) is then y [M/8][N] = (sum_i 2^i dot_i + 255 wsum) / 2
                            // and bits (optional) [M/8][Nw] its thresholded sign; else null
};

template <class ASrc, bool VEC16B, bool BITS, int WM, int WN, int FM, int FN>
__global__ __launch_bounds__(256, FM * FN >= 16 ? 1 : (FM * FN >= 8 ? 2 : 3))
void bgemm_mfma_kernel(const ASrc asrc, const uint32_t *__restrict__ B, const MfmaOut o, int M, int N,
                       int K_true, int row_dw, int tiles_m, int tiles_n, int tiles_per_xcd)
{
    static_assert(WM * WN == 4, "four waves per block");
    constexpr int BM = WM * FM * 32, BN = WN * FN * 32, KG = kMfmaKG, NT = 256;
    constexpr int STAGE_DW = KG * 4;
    // two LDS buffers: stage s + 1 is written while stage s is still being read
    __shared__ uint4 As[2][KG][BM + 1];
    __shared__ uint4 Bs[2][KG][BN + 1];
    __shared__ __align__(16) int pa_s[BM];   // set bits per A row of the tile
    __shared__ int pb_s[BN];                 // set bits per B row (= output column)

    int tm, tn;
    if (!block_to_tile(tiles_m, tiles_n, tiles_per_xcd, &tm, &tn))
        return;
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x;
    for (int i = tid; i < BM; i += NT)
        pa_s[i] = 0;
    for (int i = tid; i < BN; i += NT)
        pb_s[i] = 0;
    const int lane = tid % kWave;
    const int wave = tid / kWave;
    const int wm = (wave / WN) * (FM * 32);  // wave's row offset inside the block tile
    const int wn = (wave % WN) * (FN * 32);  // wave's column offset

    // loader: chunk idx = tid + i*NT -> (row idx / KG, k-group idx % KG); NT % KG == 0
    constexpr int A_CH = BM * KG / NT;
    constexpr int B_CH = BN * KG / NT;
    const int kg_mine = tid % KG;
    typename ASrc::Row arow[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
        arow[i] = asrc.row_nb(m0 + (tid + i * NT) / KG);
    // rows and columns beyond the matrix read the last valid one: what they produce is never stored
    const uint32_t *brow[B_CH];
#pragma unroll
    for (int i = 0; i < B_CH; ++i)
        brow[i] = B + (int64_t)min(n0 + (tid + i * NT) / KG, N - 1) * row_dw;
    uint4 pa[A_CH], pb[B_CH];
    int na[A_CH], nb[B_CH];   // set bits of the chunks this thread has fetched, per row
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
        na[i] = 0;
#pragma unroll
    for (int i = 0; i < B_CH; ++i)
        nb[i] = 0;
    bool ka[A_CH], kb_keep;   // whether a fetched chunk counts; applied when it moves to LDS, so
                              // that nothing waits for a load at the point of issue
    auto prefetch = [&](int stage) {
        const int kd = stage * STAGE_DW + kg_mine * 4;
        const typename ASrc::Step st = asrc.step(kd);
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            pa[i] = asrc.fetch_raw(arow[i], st, kd);
            ka[i] = asrc.keep(arow[i], st, kd);
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i)
            pb[i] = load_chunk_raw<VEC16B>(brow[i], kd, row_dw);
        kb_keep = kd < row_dw;
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const uint4 v = keep4(pa[i], ka[i]);
            As[buf][kg_mine][(tid + i * NT) / KG] = v;
            na[i] += popc4(v);
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            const uint4 v = keep4(pb[i], kb_keep);
            Bs[buf][kg_mine][(tid + i * NT) / KG] = v;
            nb[i] += popc4(v);
        }
    };

    // operand lane mapping of the 32x32x64 MFMA: row/column = lane % 32, k half = lane / 32
    const int lr = lane % 32, half = lane / 32;

    // thresholds and flip words of the lane's columns, fetched now so that the epilogue does not
    // start with a memory round trip (clamped: K + 1 can never be reached, tail bits stay 0)
    constexpr int NW = FN / 2;
    int lim[FN];
    uint64_t fl[NW];
    if (BITS) {
#pragma unroll
        for (int g = 0; g < FN; ++g) {
            const int col = n0 + wn + g * 32 + lr;
            lim[g] = col < N ? min(max(o.thr[col], -K_true), K_true + 1) : K_true + 1;
        }
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const int wi = ((n0 + wn) >> 6) + w;
            fl[w] = wi < o.Nw ? o.flip[wi] & valid_cols_mask(wi, N) : 0ull;
        }
    }

    v16f acc[FM][FN];
#pragma unroll
    for (int f = 0; f < FM; ++f)
#pragma unroll
        for (int g = 0; g < FN; ++g)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[f][g][r] = 0.0f;

    const int stages = (row_dw + STAGE_DW - 1) / STAGE_DW;
    prefetch(0);
    commit(0);
    __syncthreads();
    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        // the wave that has MFMAs to issue goes first; one that is fetching or handing a stage
        // over issues behind it (measured: 1 % on an 8192-cube, 2 % on the network's convolutions)
        __builtin_amdgcn_s_setprio(2);
#pragma unroll
        for (int step = 0; step < KG / 2; ++step) {
            if ((s * KG + 2 * step) * 4 >= row_dw)
                continue;                    // both k-groups of this step lie beyond the row
            const int kg = 2 * step + half;
            uint4 xa[FM], xb[FN];
#pragma unroll
            for (int f = 0; f < FM; ++f)
                xa[f] = As[buf][kg][wm + f * 32 + lr];
#pragma unroll
            for (int g = 0; g < FN; ++g)
                xb[g] = Bs[buf][kg][wn + g * 32 + lr];
            mfma_group<0, FM, FN>(xa, xb, acc);
            mfma_group<1, FM, FN>(xa, xb, acc);
            mfma_group<2, FM, FN>(xa, xb, acc);
            mfma_group<3, FM, FN>(xa, xb, acc);
            if (step == 0 && s + 1 < stages)
                prefetch(s + 1);             // global loads issued behind the first step's MFMAs
        }
        __builtin_amdgcn_s_setprio(0);
        if (s + 1 < stages)
            commit(buf ^ 1);                 // nobody reads that buffer before the barrier below
        __syncthreads();
    }

    // row popcounts: KG threads share a row, their partial counts meet in LDS
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
        atomicAdd(&pa_s[(tid + i * NT) / KG], na[i]);
#pragma unroll
    for (int i = 0; i < B_CH; ++i)
        atomicAdd(&pb_s[(tid + i * NT) / KG], nb[i]);
    __syncthreads();

    // dot = K - 2 pa - 2 pb + 4 c.  Result layout of a 32x32 block: lane -> column lane % 32;
    // register r -> row 8 * (r / 4) + 4 * (lane / 32) + r % 4.
    int kb[FN];   // K - 2 pb of the lane's columns
#pragma unroll
    for (int g = 0; g < FN; ++g)
        kb[g] = K_true - 2 * pb_s[wn + g * 32 + lr];

    if (BITS) {
        // dot >= thr  <=>  4 c + (K - 2 pb - thr) >= 2 pa  <=>  c >= pa / 2 - (K - 2 pb - thr) / 4.
        // For K < 2^20 the right-hand side is exact in fp32 (multiples of 1/4 below 2^22) and c is
        // the fp32 accumulator itself, so the decision is one add and one compare; longer K takes
        // the integer form.  The 64-lane mask of a comparison holds, for one column block, the 32
        // bits of row R (lanes 0-31) and of row R + 4 (lanes 32-63); the flip bits are XORed into
        // the masks as scalars.  Lanes 0 and 32 then drop the two rows' 64-column words (low half
        // from the even block, high half from the odd one) into the block's word table in LDS
        // (the A slabs are free by now), from where each lane picks up the words of its rows.
        constexpr int WPT = BN / 64;
        uint64_t *wt = reinterpret_cast<uint64_t *>(&As[0][0][0]);
        const bool fp_exact = K_true < (1 << 20);
        int ct[FN];
        float ctf[FN];
#pragma unroll
        for (int g = 0; g < FN; ++g) {
            ct[g] = kb[g] - lim[g];
            ctf[g] = -0.25f * (float)ct[g];
        }
        uint64_t flx[FN];   // flip bits of column block g, in both halves of a mask
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)fl[w]);
            const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(fl[w] >> 32));
            flx[2 * w] = ((uint64_t)lo << 32) | lo;
            flx[2 * w + 1] = ((uint64_t)hi << 32) | hi;
        }
        auto rows_to_table = [&](auto exact) {
#pragma unroll
            for (int f = 0; f < FM; ++f)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int4 pa4 = *reinterpret_cast<const int4 *>(&pa_s[wm + f * 32 + 8 * q + 4 * half]);
                    const int pav[4] = {pa4.x, pa4.y, pa4.z, pa4.w};
                    uint64_t mask[4][FN];
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int g = 0; g < FN; ++g) {
                            bool ge;
                            if (decltype(exact)::value)
                                ge = acc[f][g][4 * q + t] >= 0.5f * (float)pav[t] + ctf[g];
                            else
                                ge = 4 * (int)acc[f][g][4 * q + t] + ct[g] >= 2 * pav[t];
                            mask[t][g] = __ballot(ge) ^ flx[g];
                        }
                    if (lr == 0) {
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            const int row = wm + f * 32 + 8 * q + 4 * half + t;
#pragma unroll
                            for (int w = 0; w < NW; ++w) {
                                // the halves of a mask are scalars: pick one per lane with a
                                // select (a per-lane 64-bit shift of the mask costs several times that)
                                const uint64_t ml = mask[t][2 * w], mh = mask[t][2 * w + 1];
                                const uint32_t lo = half ? (uint32_t)(ml >> 32) : (uint32_t)ml;
                                const uint32_t hi = half ? (uint32_t)(mh >> 32) : (uint32_t)mh;
                                wt[row * WPT + (wn >> 6) + w] = ((uint64_t)hi << 32) | lo;
                            }
                        }
                    }
                }
        };
        if (fp_exact)
            rows_to_table(std::true_type{});
        else
            rows_to_table(std::false_type{});
        const int w0 = (n0 + wn) >> 6;
        if (o.pool_log2w == 0) {
            __builtin_amdgcn_wave_barrier();     // a wave reads back only what it wrote itself
#pragma unroll
            for (int h = 0; h < FM / 2; ++h) {     // 32 FM rows per wave, 64 lanes
                const int rl = wm + h * 64 + lane;
#pragma unroll
                for (int w = 0; w < NW; ++w)
                    if (m0 + rl < M && w0 + w < o.Nw)
                        o.bits[(int64_t)(m0 + rl) * o.Nw + w0 + w] = wt[rl * WPT + (wn >> 6) + w];
            }
        } else {
            // OR max-pool over the whole block tile
            __syncthreads();
            pool_tile_store<BM, WPT, NT>(wt, o.bits, m0, n0, M, o.Nw, o.pool_log2w, tid);
        }
    } else if (o.wsum) {
        // Bit-plane mode: the 8 planes of an input row sit in one group of 8 tile rows, planes
        // 0-3 in lanes 0-31 and planes 4-7 in lanes 32-63 of the same registers; each half adds
        // its four weighted dots and the halves meet through a lane exchange.
        const int64_t images = M >> 3;
        int ws[FN], lm[FN];
#pragma unroll
        for (int g = 0; g < FN; ++g) {
            const int col = n0 + wn + g * 32 + lr;
            ws[g] = col < N ? o.wsum[col] : 0;
            lm[g] = (o.bits && col < N) ? o.thr[col] : 0x7fffffff;   // beyond N: bit 0
        }
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int rl = wm + f * 32 + 8 * q;
                const int64_t img = (int64_t)(m0 + rl) >> 3;
                const int4 pa4 = *reinterpret_cast<const int4 *>(&pa_s[rl + 4 * half]);
                const int pav[4] = {pa4.x, pa4.y, pa4.z, pa4.w};
                int yv[FN];
#pragma unroll
                for (int g = 0; g < FN; ++g) {
                    int part = 0;
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        part += (4 * (int)acc[f][g][4 * q + t] + kb[g] - 2 * pav[t]) << (4 * half + t);
                    part += __shfl_xor(part, 32, kWave);
                    yv[g] = (part + 255 * ws[g]) / 2;          // the sum is even
                }
                if (o.C && half == 0 && img < images) {
#pragma unroll
                    for (int g = 0; g < FN; ++g) {
                        const int col = n0 + wn + g * 32 + lr;
                        if (col < N)
                            o.C[img * N + col] = yv[g];
                    }
                }
                if (o.bits) {
                    uint32_t m32[FN];
#pragma unroll
                    for (int g = 0; g < FN; ++g)
                        m32[g] = (uint32_t)__ballot(yv[g] >= lm[g]);     // both halves hold the same values
                    if (lane == 0 && img < images) {
#pragma unroll
                        for (int w = 0; w < FN / 2; ++w) {
                            const int wi = ((n0 + wn) >> 6) + w;
                            if (wi < o.Nw)
                                o.bits[img * o.Nw + wi] = (((uint64_t)m32[2 * w + 1] << 32) | m32[2 * w]) ^ (o.flip[wi] & valid_cols_mask(wi, N));
                        }
                    }
                }
            }
    } else if (o.vec_store) {
        // int32 out, 16-byte stores: a 32 x 32 block leaves the accumulators as lane -> column,
        // register -> row; it is turned through a 4 KB LDS patch of the wave's own (the A slabs
        // are free by now) so that 8 lanes write one 128-byte row segment with one store each.
        int *patch = reinterpret_cast<int *>(&As[0][0][0]) + wave * 1024;
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
            for (int g = 0; g < FN; ++g) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int4 pa4 = *reinterpret_cast<const int4 *>(&pa_s[wm + f * 32 + 8 * q + 4 * half]);
                    const int pav[4] = {pa4.x, pa4.y, pa4.z, pa4.w};
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        patch[(8 * q + 4 * half + t) * 32 + lr] = 4 * (int)acc[f][g][4 * q + t] + kb[g] - 2 * pav[t];
                }
                __builtin_amdgcn_wave_barrier();
                const int col = n0 + wn + g * 32 + 4 * (lane % 8);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int r = lane / 8 + 8 * k;
                    const int4 v = *reinterpret_cast<const int4 *>(&patch[r * 32 + 4 * (lane % 8)]);
                    const int row = m0 + wm + f * 32 + r;
                    if (row < M && col < N)     // N % 4 == 0: the four columns are inside together
                        *reinterpret_cast<int4 *>(&o.C[(int64_t)row * N + col]) = v;
                }
                __builtin_amdgcn_wave_barrier();
            }
    } else {
#pragma unroll
        for (int f = 0; f < FM; ++f)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int rl = wm + f * 32 + 8 * q + 4 * half;
                const int4 pa4 = *reinterpret_cast<const int4 *>(&pa_s[rl]);
                const int pav[4] = {pa4.x, pa4.y, pa4.z, pa4.w};
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int row = m0 + rl + t;
                    if (row >= M)
                        continue;
#pragma unroll
                    for (int g = 0; g < FN; ++g) {
                        const int col = n0 + wn + g * 32 + lr;
                        if (col < N)
                            o.C[(int64_t)row * N + col] = 4 * (int)acc[f][g][4 * q + t] + kb[g] - 2 * pav[t];
                    }
                }
            }
    }
}

// Block shapes: 2 x 2 waves of 128 x 64 (two blocks per CU) and 2 x 2 waves of 64 x 64 (three).
struct ShapeA { static constexpr int WM = 2, WN = 2, FM = 4, FN = 2; };
struct ShapeS { static constexpr int WM = 2, WN = 2, FM = 2, FN = 2; };

template <class ASrc, bool VEC16B, class S>
static int launch_mfma_shape(const ASrc &asrc, const uint32_t *b, const MfmaOut &o, int64_t M, int64_t N,
                             int64_t K_true, int64_t row_dw, hipStream_t stream)
{
    constexpr int BM = S::WM * S::FM * 32, BN = S::WN * S::FN * 32;
    const int tiles_m = (int)ceil_div(M, BM);
    const int tiles_n = (int)ceil_div(N, BN);
    const int64_t total = (int64_t)tiles_m * tiles_n;
    if (total > (1ll << 30))
        return ESP_ESHAPE;
    const int per_xcd = (int)ceil_div(total, kXcd);
    const dim3 grid((unsigned)(per_xcd * kXcd));
    if (o.bits && !o.wsum)
        hipLaunchKernelGGL((bgemm_mfma_kernel<ASrc, VEC16B, true, S::WM, S::WN, S::FM, S::FN>), grid, dim3(256), 0,
                           stream, asrc, b, o, (int)M, (int)N, (int)K_true, (int)row_dw, tiles_m, tiles_n,
                           per_xcd);
    else
        hipLaunchKernelGGL((bgemm_mfma_kernel<ASrc, VEC16B, false, S::WM, S::WN, S::FM, S::FN>), grid, dim3(256), 0,
                           stream, asrc, b, o, (int)M, (int)N, (int)K_true, (int)row_dw, tiles_m, tiles_n,
                           per_xcd);
    return launch_status();
}

template <class ASrc, bool VEC16B>
static int launch_mfma(const ASrc &asrc, const uint32_t *b, const MfmaOut &o, int64_t M, int64_t N,
                       int64_t K_true, int64_t row_dw, hipStream_t stream)
{
    // 256 x 128 blocks when they give every CU its two; otherwise 128 x 128 blocks, three per CU
    // (measured on the 512-channel convolutions at batch 256: 256 large tiles 14.5 / 21.8 us,
    // 512 small ones 12.9 / 20.6 us; with 1024 large tiles or more the large shape is faster)
    if (ceil_div(M, 256) * ceil_div(N, 128) < 512)
        return launch_mfma_shape<ASrc, VEC16B, ShapeS>(asrc, b, o, M, N, K_true, row_dw, stream);
    return launch_mfma_shape<ASrc, VEC16B, ShapeA>(asrc, b, o, M, N, K_true, row_dw, stream);
}

int bgemm_mfma_launch(const uint64_t *A, const uint64_t *B, int32_t *C, const int32_t *thr,
                      const uint64_t *flip, uint64_t *bits, int64_t M, int64_t N, int64_t K_true,
                      int64_t row_words, hipStream_t stream)
{
    if (M == 0)
        return ESP_OK;
    if (M >= (1ll << 31) || N >= (1ll << 31) || row_words >= (1ll << 29) || K_true >= kMaxMfmaK)
        return ESP_ESHAPE;
    const MfmaOut o{C, bits, thr, flip, (int)ceil_div(N, 64), 0, (N % 4 == 0) && aligned(C, 16), nullptr};
    const bool vec16 = (row_words % 2 == 0) && aligned(A, 16) && aligned(B, 16);
    const uint32_t *a = reinterpret_cast<const uint32_t *>(A);
    const uint32_t *b = reinterpret_cast<const uint32_t *>(B);
    const int row_dw = (int)(row_words * 2);
    if (vec16)
        return launch_mfma<MatrixA<true>, true>(MatrixA<true>{a, (int)M, row_dw}, b, o, M, N, K_true, row_dw,
                                                stream);
    return launch_mfma<MatrixA<false>, false>(MatrixA<false>{a, (int)M, row_dw}, b, o, M, N, K_true, row_dw,
                                              stream);
}

// Dense layer on 8-bit inputs given as bit-planes [rows][8][row_words] (Eq. 3): y and / or the
// thresholded sign bits per input row, the combination done in the product's epilogue.
int bitplane_dense_mfma_launch(const uint64_t *planes, const uint64_t *W, const int32_t *wsum, int32_t *y,
                               const int32_t *thr, const uint64_t *flip, uint64_t *bits, int64_t rows, int64_t N,
                               int64_t K_true, int64_t row_words, hipStream_t stream)
{
    const int64_t M = rows * 8;
    if (M >= (1ll << 31) || N >= (1ll << 31) || row_words >= (1ll << 29) || K_true >= (1 << 21))
        return ESP_ESHAPE;        // 2 * 255 * K must stay inside int32
    const MfmaOut o{y, bits, thr, flip, (int)ceil_div(N, 64), 0, 0, wsum};
    const bool vec16 = (row_words % 2 == 0) && aligned(planes, 16) && aligned(W, 16);
    const uint32_t *a = reinterpret_cast<const uint32_t *>(planes);
    const uint32_t *b = reinterpret_cast<const uint32_t *>(W);
    const int row_dw = (int)(row_words * 2);
    if (vec16)
        return launch_mfma<MatrixA<true>, true>(MatrixA<true>{a, (int)M, row_dw}, b, o, M, N, K_true, row_dw,
                                                stream);
    return launch_mfma<MatrixA<false>, false>(MatrixA<false>{a, (int)M, row_dw}, b, o, M, N, K_true, row_dw,
                                              stream);
}

int bconv_mfma_launch(const uint64_t *in, const uint64_t *filt, int32_t *C_out, const int32_t *thr,
                      const uint64_t *flip, uint64_t *bits_out, int B, int H, int W, int C, int L2,
                      int kh, int kw, int stride, int pad, int H2, int W2, int pool_log2w, hipStream_t stream)
{
    const int64_t M = (int64_t)B * H2 * W2;
    const int64_t K_true = (int64_t)kh * kw * C;
    if (M >= (1ll << 31) || K_true >= kMaxMfmaK || (int64_t)B * H * W * (C / 32) >= (1ll << 40))
        return ESP_ESHAPE;
    const ConvA a = make_conv_a(in, B, H, W, C, kh, kw, stride, pad, H2, W2);
    const MfmaOut o{C_out, bits_out, thr, flip, (int)ceil_div(L2, 64), pool_log2w, (L2 % 4 == 0) && aligned(C_out, 16), nullptr};
    return launch_mfma<ConvA, true>(a, reinterpret_cast<const uint32_t *>(filt), o, M, L2, K_true, a.row_dw,
                                    stream);
}

} // namespace esp

extern "C" int esp_bgemm_mfma(const uint64_t *A, const uint64_t *B, int32_t *C,
                              int64_t M, int64_t N, int64_t K, esp_stream stream)
{
    using namespace esp;
    if (M < 0 || N <= 0 || K <= 0)
        return ESP_EINVAL;
    if (K >= kMaxMfmaK)
        return ESP_ESHAPE;
    if (M == 0)
        return ESP_OK;
    if (!A || !B || !C)
        return ESP_EINVAL;
    if (!aligned(A, 8) || !aligned(B, 8) || !aligned(C, 4))
        return ESP_EALIGN;
    return bgemm_mfma_launch(A, B, C, nullptr, nullptr, nullptr, M, N, K, ceil_div(K, 64), as_stream(stream));
}
