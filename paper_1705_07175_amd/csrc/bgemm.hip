// Binary matrix product on packed words (Sec. 4.2, Eq. 2 of arXiv 1705.07175):
//   C[m][n] = K - 2 * sum_w popcount(A[m][w] XOR B[n][w]).
//
// Four kernels:
//  * bgemm_tile_kernel  -- compute-bound case.  A block stages BM x 1024-bit and
//    BN x 1024-bit slabs of the packed rows in LDS as 16-byte k-groups, every lane
//    keeps a TM x TN tile of int32 mismatch counters in registers and runs a pure
//    v_xor_b32 / v_bcnt_u32_b32 (accumulating popcount) inner loop on 32-bit halves
//    of the words.  Two LDS stage buffers (one barrier per stage), global loads one
//    stage ahead, LDS operand reads one k-group ahead: every wave runs at its own fixed
//    pace, so what it waits for is lost unless another wave of its SIMD fills the gap
//    (8 x 4 counters per lane leave room for three waves per SIMD, 8 x 8 for two).
//    The paper's own design (shared-memory tiles + register blocking, Sec. 5.2
//    "Efficient Matrix multiplication") is kept; tile shapes, the LDS layout and the
//    block order are chosen for 64-wide wavefronts and 8 XCDs.
//    The A operand comes either from a packed matrix or, for convolutions, straight
//    from the packed NHWC input (the unrolling of Sec. 5.2 / Fig. 3 done by the
//    loader: the lowered matrix never exists in memory).  The epilogue writes either
//    the int32 dot products or, with the folded batch-norm threshold, the packed
//    sign bits of the next layer (the bit-packing sign activation of Sec. 6.3).
//  * bgemv_kernel       -- small M (matrix-vector, Sec. 6.2 "Optimized kernels"):
//    bandwidth-bound streaming of B with the few A rows held in LDS; also used with
//    the operands swapped for products with few columns (the 10 scores of a network).
//  * bgemv_bits_kernel  -- the same with the threshold + sign + pack epilogue.
//  * bfew_bits_kernel   -- products of a few hundred rows (a network's convolutions at
//    batch 1): lane = row, K split over the waves of a block, threshold epilogue.
#include "esp_internal.h"
#include "tile_sources.h"
#include "tile_epilogues.h"

namespace esp {

// ---------------------------------------------------------------------------------
// Tiled kernel
// ---------------------------------------------------------------------------------
constexpr int kKG = 8;        // 16-byte k-groups per LDS stage: 8 * 128 bits = 1024 bits of K
constexpr int kStageDw = 32;  // dwords of K per row per stage

template <int BM, int BN, int TM, int TN, class ASrc, bool VEC16B, bool BITS>
__global__ __launch_bounds__((BM / TM) * (BN / TN))
void bgemm_tile_kernel(const ASrc asrc, const uint32_t *__restrict__ B, const StoreDots dots,
                       const StoreSignBits bits, int M, int N, int K_true, int row_dw,
                       int tiles_m, int tiles_n, int tiles_per_xcd)
{
    constexpr int TX = BN / TN;      // threads along N
    constexpr int TY = BM / TM;      // threads along M
    constexpr int NT = TX * TY;
    static_assert(TN % 4 == 0, "columns are owned in groups of four");
    static_assert((BM * kKG) % NT == 0 && (BN * kKG) % NT == 0, "loader shape");

    // two stage buffers: stage s + 1 is written while other waves still read stage s, so one
    // barrier per stage is enough
    __shared__ uint4 As[2][kKG][BM + 1];
    __shared__ uint4 Bs[2][kKG][BN + 1];

    int tm, tn;
    if (!block_to_tile(tiles_m, tiles_n, tiles_per_xcd, &tm, &tn))
        return;
    const int m0 = tm * BM;
    const int n0 = tn * BN;

    const int tid = threadIdx.x;
    const int tx = tid % TX;
    const int ty = tid / TX;

    // loader: chunk idx = tid + i*NT covers (row idx / kKG, k-group idx % kKG); NT is a
    // multiple of kKG, so a thread always loads the same k-group of its rows.  Loads are
    // branch-free (clamped rows, masked K tail): rows beyond M or N compute values that are
    // never stored.
    constexpr int A_CH = BM * kKG / NT;
    constexpr int B_CH = BN * kKG / NT;
    const int kg_mine = tid % kKG;
    typename ASrc::Row arow[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i)
        arow[i] = asrc.row_nb(m0 + (tid + i * NT) / kKG);
    const uint32_t *brow[B_CH];
#pragma unroll
    for (int i = 0; i < B_CH; ++i)
        brow[i] = B + (int64_t)min(n0 + (tid + i * NT) / kKG, N - 1) * row_dw;
    uint4 pa[A_CH], pb[B_CH];
    bool ka[A_CH], kb;     // whether a chunk counts; applied when it moves to LDS
    bool whole;            // the fetched stage has no K tail

    auto prefetch = [&](int stage) {
        const int kd = stage * kStageDw + kg_mine * 4;
        const typename ASrc::Step st = asrc.step(kd);
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            pa[i] = asrc.fetch_raw(arow[i], st, kd);
            ka[i] = asrc.keep(arow[i], st, kd);
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i)
            pb[i] = load_chunk_raw<VEC16B>(brow[i], kd, row_dw);
        kb = kd < row_dw;
        whole = (stage + 1) * kStageDw <= row_dw;
    };

    // A stage of a packed-matrix product that lies inside the rows altogether (uniform over the
    // block) needs no K-tail mask; a gathered A masks its border pixels in every stage.
    auto commit = [&](int buf) {
        auto store_b = [&](int i, const uint4 v) {
            const int nl = (tid + i * NT) / kKG;
            // column nl is register column j of lane tx: nl = (j/4)*(4*TX) + tx*4 + j%4
            const int j = (nl / (4 * TX)) * 4 + nl % 4;
            Bs[buf][kg_mine][j * TX + (nl % (4 * TX)) / 4] = v;
        };
        if (!ASrc::kGathered && whole) {       // uniform over the block
#pragma unroll
            for (int i = 0; i < A_CH; ++i)
                As[buf][kg_mine][(tid + i * NT) / kKG] = pa[i];
#pragma unroll
            for (int i = 0; i < B_CH; ++i)
                store_b(i, pb[i]);
        } else {
#pragma unroll
            for (int i = 0; i < A_CH; ++i)
                As[buf][kg_mine][(tid + i * NT) / kKG] = keep4(pa[i], ka[i]);
#pragma unroll
            for (int i = 0; i < B_CH; ++i)
                store_b(i, keep4(pb[i], kb));
        }
    };

    int acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            acc[i][j] = 0;

    // thresholds of the lane's columns.  The small tiles serve products whose time is a chain
    // of memory latencies, so they fetch them now, alongside the first stage, and keep them in
    // registers; the large tiles need their registers for the main loop: their limits and flip
    // words are fetched now as well, but wait in LDS for the epilogue, which then starts
    // without a trip to memory.
    constexpr bool kEarlyLimits = BITS && TM < 8;
    int lim[BITS ? TN : 1];
    __shared__ __align__(16) int lim_s[(BITS && !kEarlyLimits) ? BN : 4];
    __shared__ uint64_t flip_s[(BITS && !kEarlyLimits) ? BN / 64 : 1];
    if constexpr (kEarlyLimits) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
            lim[j] = bits.mismatch_limit(n0 + (j / 4) * 4 * TX + tx * 4 + j % 4, N, K_true);
    } else if constexpr (BITS) {
        for (int c = tid; c < BN; c += NT)
            lim_s[c] = bits.mismatch_limit(n0 + c, N, K_true);
        if (tid < BN / 64)
            flip_s[tid] = (n0 >> 6) + tid < bits.Nw ? bits.flip[(n0 >> 6) + tid] & valid_cols_mask((n0 >> 6) + tid, N) : 0ull;
    }

    const int stages = (row_dw + kStageDw - 1) / kStageDw;
    prefetch(0);
    commit(0);
    __syncthreads();
    for (int s = 0; s < stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < stages)
            prefetch(s + 1);
        const int left_dw = row_dw - s * kStageDw;
        const int kgs = left_dw >= kStageDw ? kKG : (left_dw + 3) / 4;
        // Operands travel LDS -> registers one k-group ahead of their use: while k-group kg is
        // counted, the B chunks and the first A chunk of k-group kg + 1 arrive, and the other
        // A chunks of kg (issued at its start) are not needed before its second row of
        // counters.  A wave that waits for LDS leaves its SIMD to the other wave, which cannot
        // make up for it, so no counter should ever wait.  Two register sets alternate.
        auto kgroup = [&](int kg, int kg_next, const uint4 &a0, const uint4 (&b)[TN], uint4 &a0_next,
                          uint4 (&b_next)[TN]) {
            uint4 a[TM];
            a[0] = a0;
#pragma unroll
            for (int i = 1; i < TM; ++i)
                a[i] = As[buf][kg][ty + TY * i];
            a0_next = As[buf][kg_next][ty];
            // first row of counters on operands that arrived during the previous k-group; the
            // reads of b_next are issued behind it so that no more than 15 reads are ever
            // outstanding (the wait counter cannot express more, and would wait too early)
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                xor_popc_acc4(acc[0][j], a[0], b[j]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b_next[j] = Bs[buf][kg_next][j * TX + tx];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 1; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    xor_popc_acc4(acc[i][j], a[i], b[j]);
        };
        uint4 a0_even, b_even[TN], a0_odd, b_odd[TN];
        a0_even = As[buf][0][ty];
#pragma unroll
        for (int j = 0; j < TN; ++j)
            b_even[j] = Bs[buf][0][j * TX + tx];
        int kg = 0;
        for (; kg + 1 < kgs; kg += 2) {
            kgroup(kg, kg + 1, a0_even, b_even, a0_odd, b_odd);
            kgroup(kg + 1, min(kg + 2, kKG - 1), a0_odd, b_odd, a0_even, b_even);
        }
        if (kg < kgs)
            kgroup(kg, kg, a0_even, b_even, a0_odd, b_odd);
        if (s + 1 < stages)
            commit(buf ^ 1);
        __syncthreads();
    }

    // Epilogue: dot = K - 2 * mismatches.
    if constexpr (BITS) {
        static_assert(TX == 16, "a 64-column word is spread over 16 lanes x 4 columns");
        if constexpr (!kEarlyLimits) {
#pragma unroll
            for (int jg = 0; jg < TN / 4; ++jg) {
                const int4 l4 = *reinterpret_cast<const int4 *>(&lim_s[jg * 4 * TX + tx * 4]);
                lim[jg * 4 + 0] = l4.x;
                lim[jg * 4 + 1] = l4.y;
                lim[jg * 4 + 2] = l4.z;
                lim[jg * 4 + 3] = l4.w;
            }
        }
        LaneWord lw;
        if constexpr (TM == 8 && TN == 8)
            lw = bits.template tile<TY>(acc, lim, tx, ty);
        else if constexpr (TM == 8)
            lw = bits.template tile_8x4<TY>(acc, lim, tx, ty);
        else
            lw = bits.template tile<TY, TM>(acc, lim, tx, ty);
        const int w = (n0 >> 6) + lw.wl;
        uint64_t word;
        if constexpr (kEarlyLimits)
            word = bits.finish(lw, w);
        else
            word = lw.have ? ((((uint64_t)lw.hi << 32) | lw.lo) ^ flip_s[lw.wl]) : 0ull;   // flip_s is 0 beyond Nw
        if (bits.pool_log2w == 0) {
            if (lw.have && m0 + lw.rl < M && w < bits.Nw)
                bits.out[(int64_t)(m0 + lw.rl) * bits.Nw + w] = word;
        } else {
            // 2x2 max-pool of +-1 values = OR of the sign bits: the tile's words meet in LDS
            // (the A slab is free after the last stage) and every pooled word ORs its four sources
            constexpr int WPT = BN / 64;
            uint64_t *wt = reinterpret_cast<uint64_t *>(&As[0][0][0]);
            if (lw.have)
                wt[lw.rl * WPT + lw.wl] = word;
            __syncthreads();
            pool_tile_store<BM, WPT, NT>(wt, bits.out, m0, n0, M, bits.Nw, bits.pool_log2w, tid);
        }
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = m0 + ty + TY * i;
            if (r < M)
                dots.template row<TN, TX>(r, N, K_true, n0, tx, acc[i]);
        }
    }
}

// What the epilogue of a tiled launch produces.
struct TileOut {
    int32_t *C = nullptr;            // int32 dots [M][N]            (BITS == false)
    uint64_t *bits = nullptr;        // packed signs [M][ceil(N/64)] (BITS == true)
    const int32_t *thr = nullptr;
    const uint64_t *flip = nullptr;
    int pool_log2w = 0;              // fused 2x2 max-pool behind the sign: log2 of the conv's W2
};

template <int BM, int BN, int TM, int TN, class ASrc, bool VEC16B>
static int launch_tile2(const ASrc &asrc, const uint32_t *b, const TileOut &o, int64_t M, int64_t N,
                        int64_t K_true, int64_t row_dw, hipStream_t stream)
{
    const int tiles_m = (int)ceil_div(M, BM);
    const int tiles_n = (int)ceil_div(N, BN);
    const int64_t total = (int64_t)tiles_m * tiles_n;
    if (total > (1ll << 30))
        return ESP_ESHAPE;
    const int per_xcd = (int)ceil_div(total, kXcd);
    const dim3 grid((unsigned)(per_xcd * kXcd));
    const dim3 block((BM / TM) * (BN / TN));
    const StoreDots dots{o.C, (N % 4 == 0) && aligned(o.C, 16)};
    const StoreSignBits bits{o.bits, o.thr, o.flip, (int)ceil_div(N, 64), (int)N, o.pool_log2w};
    if (o.bits)
        hipLaunchKernelGGL((bgemm_tile_kernel<BM, BN, TM, TN, ASrc, VEC16B, true>), grid, block, 0, stream,
                           asrc, b, dots, bits, (int)M, (int)N, (int)K_true, (int)row_dw, tiles_m, tiles_n,
                           per_xcd);
    else
        hipLaunchKernelGGL((bgemm_tile_kernel<BM, BN, TM, TN, ASrc, VEC16B, false>), grid, block, 0, stream,
                           asrc, b, dots, bits, (int)M, (int)N, (int)K_true, (int)row_dw, tiles_m, tiles_n,
                           per_xcd);
    return launch_status();
}

// Tile shape.  Every CU should get at least two blocks: 128x128 (8x8 counters per lane, two
// waves per SIMD) or 128x64 (8x4, three waves per SIMD) while 512 of them exist, otherwise
// 64x64 (4x4) or 32x64, which keep small-N / small-M products spread out.  Between the two
// large shapes the source of A decides (measured): rows of a packed matrix are cheap to fetch
// and the narrower tile, whose third wave fills the other two's waits, is 2.5 % faster on an
// 8192-cube; rows gathered from an NHWC input cost address arithmetic per row and stage, and a
// tile half as wide fetches every row twice as often (3-7 % slower on 3x3 convolutions over
// 256 and 512 channels).
template <class ASrc, bool VEC16B>
static int launch_tile(const ASrc &asrc, const uint32_t *b, const TileOut &o, int64_t M, int64_t N,
                       int64_t K_true, int64_t row_dw, hipStream_t stream)
{
    // a fused 2x2 pool needs whole pairs of image rows in a tile: BM a multiple of 2 * W2
    const int quantum = o.pool_log2w ? 2 << o.pool_log2w : 1;
    const int64_t big_tiles = ceil_div(M, 128) * ceil_div(N, 128);
    const bool narrow_fills = ceil_div(M, 128) * ceil_div(N, 64) >= 512;
    if constexpr (ASrc::kGathered) {     // (only convolutions pool, so quantum is 1 otherwise)
        if (big_tiles >= 512 || quantum > 64)
            return launch_tile2<128, 128, 8, 8, ASrc, VEC16B>(asrc, b, o, M, N, K_true, row_dw, stream);
    }
    // 768 of the 128 x 64 tiles are resident at once (three per compute unit).  Between one and six
    // such rounds the partly filled last round costs more than the smaller tile's extra LDS traffic:
    // products of packed matrices then take 64 x 64 tiles (measured on squares: 12 % faster at 1.5
    // rounds, 8 % at 2.04, 1 % at 2.7, 3 % at 4.2; 1 % slower from 6 rounds on and below one round).
    const int64_t narrow_tiles = ceil_div(M, 128) * ceil_div(N, 64);
    const bool few_rounds = !ASrc::kGathered && quantum == 1 && narrow_tiles > 768 && narrow_tiles < 6 * 768;
    if (narrow_fills && !few_rounds)
        return launch_tile2<128, 64, 8, 4, ASrc, VEC16B>(asrc, b, o, M, N, K_true, row_dw, stream);
    // small products (dense layers at moderate batch, convolutions at batch 1): halve the
    // rows per lane so that twice as many waves share the work when the chip is not full
    if (ceil_div(M, 64) * ceil_div(N, 64) >= 256 || quantum > 32)
        return launch_tile2<64, 64, 4, 4, ASrc, VEC16B>(asrc, b, o, M, N, K_true, row_dw, stream);
    return launch_tile2<32, 64, 2, 4, ASrc, VEC16B>(asrc, b, o, M, N, K_true, row_dw, stream);
}

// ---------------------------------------------------------------------------------
// Few-rows kernel with the threshold epilogue (the convolutions and dense layers of a network
// evaluated one image at a time, Sec. 6.2 / 6.3: M is a few hundred rows at most).  The tiled
// kernel would give such a product 16-32 blocks whose lanes each walk all of K; here the work
// is spread the other way round:
//  * a wave owns 64 rows of A, lane = row, and kNB = 8 rows of B whose 16-byte chunks are the
//    same for every lane (uniform addresses: they travel through the scalar data path and
//    enter the XOR as scalar operands);
//  * the waves of a block split K: wave w takes chunks w, w + W, ..., and the per-lane
//    mismatch counts of the W waves meet in LDS;
//  * 8 columns = one byte of the packed output row; the grid covers every byte of every word
//    (columns beyond N give zero bits);
//  * a fused 2x2 max-pool ORs the bytes of lanes l, l^1, l^W2, l^(W2+1) (64 rows are whole
//    pairs of image rows when W2 <= 32).
// ---------------------------------------------------------------------------------
constexpr int kFewNB = 8;

template <class ASrc>
__global__ __launch_bounds__(1024)
void bfew_bits_kernel(const ASrc asrc, const uint32_t *__restrict__ B, const int32_t *__restrict__ thr,
                      const uint64_t *__restrict__ flip, uint8_t *__restrict__ out, int M, int N,
                      int K_true, int row_dw, int pool_log2w)
{
    constexpr int NB = kFewNB;
    __shared__ int red[NB][kWave];
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int W = blockDim.x / kWave;
    const int m0 = blockIdx.x * kWave;
    const int piece = blockIdx.y;            // byte of the packed output row
    const int n0 = piece * NB;
    for (int i = threadIdx.x; i < NB * kWave; i += blockDim.x)
        (&red[0][0])[i] = 0;

    const typename ASrc::Row arow = asrc.row_nb(m0 + lane);
    const uint32_t *brow[NB];                // uniform; rows beyond N read the last row
#pragma unroll
    for (int j = 0; j < NB; ++j)
        brow[j] = B + (int64_t)min(n0 + j, N - 1) * row_dw;
    int acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
        acc[j] = 0;
    const int nch = row_dw / 4;
    for (int c = wave; c < nch; c += W) {
        const int kd = c * 4;
        const uint4 a = asrc.fetch_nb(arow, asrc.step(kd), kd);
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const uint4 b = *reinterpret_cast<const uint4 *>(brow[j] + kd);
            acc[j] += __popc(a.x ^ b.x) + __popc(a.y ^ b.y) + __popc(a.z ^ b.z) + __popc(a.w ^ b.w);
        }
    }
    __syncthreads();                         // red is zero
    if (W > 1) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
            atomicAdd(&red[j][lane], acc[j]);
        __syncthreads();
    }
    if (wave != 0)
        return;
    uint32_t byte = 0;
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int n = n0 + j;
        const int a = W > 1 ? red[j][lane] : acc[j];
        // dot = K - 2a >= thr  <=>  a <= floor((K - thr) / 2); columns beyond N: bit 0
        const int t = min(max(thr[min(n, N - 1)], -K_true), K_true + 1);
        byte |= (n < N && a <= ((K_true - t) >> 1)) ? 1u << j : 0u;
    }
    byte ^= (uint32_t)((flip[piece / 8] & valid_cols_mask(piece / 8, N)) >> (8 * (piece % 8))) & 0xffu;
    const int pieces = gridDim.y;            // bytes per packed output row
    const int r = m0 + lane;
    if (pool_log2w == 0) {
        if (r < M)
            out[(int64_t)r * pieces + piece] = (uint8_t)byte;
        return;
    }
    const int W2 = 1 << pool_log2w;
    byte |= (uint32_t)__shfl_xor((int)byte, 1, kWave);
    byte |= (uint32_t)__shfl_xor((int)byte, W2, kWave);
    if ((lane & 1) == 0 && (lane & W2) == 0 && r < M) {
        const int line = r >> pool_log2w, n = r & (W2 - 1);
        const int64_t prow = (int64_t)(line >> 1) * (W2 >> 1) + (n >> 1);
        out[prow * pieces + piece] = (uint8_t)byte;
    }
}

// Does the few-rows kernel apply?  Rows that the tiled kernel's smallest tiles would spread
// over less than one block per CU, 16-byte chunks, and (pooled) whole row pairs in 64 rows.
static bool few_rows_ok(int64_t M, int64_t N, int64_t row_dw, int pool_log2w)
{
    return ceil_div(M, 32) * ceil_div(N, 64) < 256 && row_dw % 4 == 0 && row_dw / 4 < (1 << 20) &&
           ceil_div(M, 64) < 65536 && ceil_div(N, 64) * 8 < 65536 && (pool_log2w == 0 || pool_log2w <= 5);
}

template <class ASrc>
static int launch_few(const ASrc &asrc, const uint32_t *b, const TileOut &o, int64_t M, int64_t N,
                      int64_t K_true, int64_t row_dw, hipStream_t stream)
{
    const int64_t nch = row_dw / 4;
    const dim3 grid((unsigned)ceil_div(M, 64), (unsigned)(ceil_div(N, 64) * 8));
    // The waves of a block split K: up to 16 while every CU gets at most one block.  A CU holds
    // 28 waves of this kernel (its 103 scalar registers allow 7 per SIMD), i.e. one block of 16
    // waves but three of 8: with more blocks than CUs, 8 waves keep all of them resident instead of
    // running two rounds (256 x 1024 x 8192: 10.2 -> 8.7 us, 64 x 4096 x 4096: 7.9 -> 6.4 us; grids
    // of at most 256 blocks lose 5-30 % with 8).
    const int wmax = (int64_t)grid.x * grid.y > 256 ? 8 : 16;
    const int waves = (int)(nch < wmax ? nch : wmax);
    const dim3 block((unsigned)(waves * kWave));
    hipLaunchKernelGGL((bfew_bits_kernel<ASrc>), grid, block, 0, stream, asrc, b, o.thr, o.flip,
                       reinterpret_cast<uint8_t *>(o.bits), (int)M, (int)N, (int)K_true, (int)row_dw,
                       o.pool_log2w);
    return launch_status();
}

static int tile_matrix(const uint64_t *A, const uint64_t *B, const TileOut &o, int64_t M, int64_t N,
                       int64_t K_true, int64_t row_words, hipStream_t stream)
{
    const bool vec16 = (row_words % 2 == 0) && aligned(A, 16) && aligned(B, 16);
    const uint32_t *a = reinterpret_cast<const uint32_t *>(A);
    const uint32_t *b = reinterpret_cast<const uint32_t *>(B);
    const int row_dw = (int)(row_words * 2);
    if (vec16 && o.bits && few_rows_ok(M, N, row_dw, 0))
        return launch_few(MatrixA<true>{a, (int)M, row_dw}, b, o, M, N, K_true, row_dw, stream);
    if (vec16)
        return launch_tile<MatrixA<true>, true>(MatrixA<true>{a, (int)M, row_dw}, b, o, M, N, K_true,
                                                row_dw, stream);
    return launch_tile<MatrixA<false>, false>(MatrixA<false>{a, (int)M, row_dw}, b, o, M, N, K_true,
                                              row_dw, stream);
}

// ---------------------------------------------------------------------------------
// Small-M kernel: stream B once, A (at most MS rows) sits in LDS.
// A wave splits into 64/LPR groups of LPR lanes; each group owns one row of B at a
// time, its lanes stride over the row's chunks, and a butterfly over the group's lanes
// sums the per-lane mismatch counts.
// ---------------------------------------------------------------------------------
template <bool VEC16> struct Chunk;
template <> struct Chunk<true> {
    using type = uint4;
    static constexpr int words = 2;
    static __device__ __forceinline__ int mism(const uint4 a, const uint4 b)
    {
        return __popc(a.x ^ b.x) + __popc(a.y ^ b.y) + __popc(a.z ^ b.z) + __popc(a.w ^ b.w);
    }
    static __device__ __forceinline__ uint4 zero() { return make_uint4(0u, 0u, 0u, 0u); }
};
template <> struct Chunk<false> {
    using type = uint2;
    static constexpr int words = 1;
    static __device__ __forceinline__ int mism(const uint2 a, const uint2 b)
    {
        return __popc(a.x ^ b.x) + __popc(a.y ^ b.y);
    }
    static __device__ __forceinline__ uint2 zero() { return make_uint2(0u, 0u); }
};

template <int MS, bool VEC16, bool A_LDS, bool PRE>
__global__ __launch_bounds__(256)
void bgemv_kernel(const uint64_t *__restrict__ A, const uint64_t *__restrict__ B,
                  int32_t *__restrict__ C, int M, int N, int K_true, int row_words, int lpr,
                  int groups_per_wave, int64_t c_stride_m, int64_t c_stride_row)
{
    using CK = Chunk<VEC16>;
    using chunk_t = typename CK::type;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    chunk_t *As = reinterpret_cast<chunk_t *>(smem_raw);

    const int nch = row_words / CK::words;
    const chunk_t *Ag = reinterpret_cast<const chunk_t *>(A);
    const chunk_t *Bg = reinterpret_cast<const chunk_t *>(B);

    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int waves_per_block = blockDim.x / kWave;
    const int rpw = kWave / lpr;          // rows of B per wave pass
    const int sub = lane / lpr;           // which of those rows this lane works on
    const int cl = lane % lpr;            // lane index within the row group
    const int64_t groups = ((int64_t)N + rpw - 1) / rpw;
    // a block owns a contiguous run of rows, so that the blocks in flight sweep B as one front
    const int64_t g0 = ((int64_t)blockIdx.x * waves_per_block + wave) * groups_per_wave;

    // PRE (one row group per wave: a product whose time is a chain of latencies): the weights
    // are the long pole, so the first loads of the wave's row go out before A is staged (rows
    // beyond N read row N - 1; their results are not stored)
    chunk_t pre0 = CK::zero(), pre1 = CK::zero();
    if (PRE) {
        const int64_t row = min(g0 * rpw + sub, (int64_t)N - 1);
        const chunk_t *brow = Bg + row * nch;
        if (cl < nch)
            pre0 = brow[cl];
        if (cl + lpr < nch)
            pre1 = brow[cl + lpr];
    }
    if (A_LDS) {
        for (int i = threadIdx.x; i < MS * nch; i += blockDim.x)
            As[i] = (i / nch < M) ? Ag[i] : CK::zero();
        __syncthreads();
    }

    for (int64_t g = g0; g < g0 + groups_per_wave && g < groups; ++g) {
        const int64_t row = g * rpw + sub;
        const bool valid = row < N;
        int acc[MS];
#pragma unroll
        for (int m = 0; m < MS; ++m)
            acc[m] = 0;
        const chunk_t *brow = Bg + row * nch;
        int c = cl;
        // two chunks per trip keep more loads in flight
        for (; c + lpr < nch; c += 2 * lpr) {
            const bool first = PRE && g == g0 && c == cl;
            const chunk_t b0 = first ? pre0 : (valid ? brow[c] : CK::zero());
            const chunk_t b1 = first ? pre1 : (valid ? brow[c + lpr] : CK::zero());
#pragma unroll
            for (int m = 0; m < MS; ++m) {
                const chunk_t a0 = A_LDS ? As[m * nch + c] : (m < M ? Ag[m * nch + c] : CK::zero());
                const chunk_t a1 = A_LDS ? As[m * nch + c + lpr]
                                         : (m < M ? Ag[m * nch + c + lpr] : CK::zero());
                acc[m] += CK::mism(a0, b0) + CK::mism(a1, b1);
            }
        }
        if (c < nch) {
            const bool first = PRE && g == g0 && c == cl;
            const chunk_t b0 = first ? pre0 : (valid ? brow[c] : CK::zero());
#pragma unroll
            for (int m = 0; m < MS; ++m) {
                const chunk_t a0 = A_LDS ? As[m * nch + c] : (m < M ? Ag[m * nch + c] : CK::zero());
                acc[m] += CK::mism(a0, b0);
            }
        }
        for (int off = lpr >> 1; off > 0; off >>= 1) {
#pragma unroll
            for (int m = 0; m < MS; ++m)
                acc[m] += __shfl_xor(acc[m], off, kWave);
        }
        if (valid && cl == 0) {
#pragma unroll
            for (int m = 0; m < MS; ++m)
                if (m < M)
                    C[m * c_stride_m + row * c_stride_row] = K_true - 2 * acc[m];
        }
    }
}

constexpr size_t kGemvLdsBytes = 64 * 1024;
constexpr int kGemvMaxM = 8;   // rows of A the small-M kernels take

// C[m * c_stride_m + n * c_stride_row] = dot(A row m, B row n): strides (N, 1) for the plain
// product, (1, M') when the caller has swapped the operands of a product with few columns.
template <int MS, bool VEC16>
static int launch_gemv2(const uint64_t *A, const uint64_t *B, int32_t *C, int64_t M, int64_t N,
                        int64_t K_true, int64_t row_words, int64_t c_stride_m, int64_t c_stride_row,
                        hipStream_t stream)
{
    const int nch = (int)(row_words / (VEC16 ? 2 : 1));
    int lpr = 1;
    while (lpr < kWave && lpr < nch)
        lpr <<= 1;
    const int rpw = kWave / lpr;
    const int64_t groups = ceil_div(N, rpw);
    // Several row groups per wave amortise the copy of A into LDS, as long as the grid still
    // has a few thousand blocks to spread over 256 CUs.
    // (Measured on a 1 GiB B: 1 group per wave 4.3 TB/s, 4 groups 5.9 TB/s, 16 groups 5.6 TB/s.)
    int gpw = (int)(groups / (4 * 8192));
    gpw = gpw < 1 ? 1 : (gpw > 4 ? 4 : gpw);
    const unsigned grid = grid_for(groups, 4 /* waves per block */ * gpw);
    const size_t lds = (size_t)MS * row_words * 8;
    if (lds <= kGemvLdsBytes && gpw == 1)
        hipLaunchKernelGGL((bgemv_kernel<MS, VEC16, true, true>), dim3(grid), dim3(256), lds, stream, A, B, C,
                           (int)M, (int)N, (int)K_true, (int)row_words, lpr, gpw, c_stride_m, c_stride_row);
    else if (lds <= kGemvLdsBytes)
        hipLaunchKernelGGL((bgemv_kernel<MS, VEC16, true, false>), dim3(grid), dim3(256), lds, stream, A, B, C,
                           (int)M, (int)N, (int)K_true, (int)row_words, lpr, gpw, c_stride_m, c_stride_row);
    else
        hipLaunchKernelGGL((bgemv_kernel<MS, VEC16, false, false>), dim3(grid), dim3(256), 0, stream, A, B, C,
                           (int)M, (int)N, (int)K_true, (int)row_words, lpr, gpw, c_stride_m, c_stride_row);
    return launch_status();
}

template <int MS>
static int launch_gemv(const uint64_t *A, const uint64_t *B, int32_t *C, int64_t M, int64_t N,
                       int64_t K_true, int64_t row_words, hipStream_t stream, bool swapped = false)
{
    const bool vec16 = (row_words % 2 == 0) && aligned(A, 16) && aligned(B, 16);
    const int64_t sm = swapped ? 1 : N, sr = swapped ? M : 1;
    return vec16 ? launch_gemv2<MS, true>(A, B, C, M, N, K_true, row_words, sm, sr, stream)
                 : launch_gemv2<MS, false>(A, B, C, M, N, K_true, row_words, sm, sr, stream);
}

// ---------------------------------------------------------------------------------
// Small-M product with the folded batch-norm threshold + sign in the epilogue (one image at
// a time, Sec. 6.2 "Optimized kernels"): a block owns RB = 64 or 16 consecutive rows of B,
// i.e. one packed output word, or one 16-bit quarter of it, per row of A, so no int32 score
// and no second launch is needed (16 rows when 64 would leave most CUs without a block).
// The block's waves split the rows; inside a wave lpr lanes share a row as in bgemv_kernel,
// and every lane keeps PASSES rows in flight (waves * PASSES * 64 / lpr == RB).
// ---------------------------------------------------------------------------------
template <int MS, bool VEC16, int PASSES>
__global__ __launch_bounds__(1024)
void bgemv_bits_kernel(const uint64_t *__restrict__ A, const uint64_t *__restrict__ B,
                       const int32_t *__restrict__ thr, const uint64_t *__restrict__ flip,
                       uint64_t *__restrict__ out, int M, int N, int K_true, int row_words, int lpr, int RB)
{
    using CK = Chunk<VEC16>;
    using chunk_t = typename CK::type;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    chunk_t *As = reinterpret_cast<chunk_t *>(smem_raw);
    __shared__ unsigned char decided[MS][64];   // (m, row of the block) -> dot >= thr

    const int nch = row_words / CK::words;
    const chunk_t *Ag = reinterpret_cast<const chunk_t *>(A);
    const chunk_t *Bg = reinterpret_cast<const chunk_t *>(B);

    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    const int rpw = kWave / lpr;          // rows of B per wave pass
    const int sub = lane / lpr;
    const int cl = lane % lpr;
    const int n_blk = blockIdx.x * RB;
    // row handled in pass p: the wave owns PASSES * rpw consecutive rows
    const int row0 = n_blk + wave * (PASSES * rpw) + sub;

    // the weights are the long pole: start on them before A is staged
    chunk_t b[PASSES];
    int t[PASSES];
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int row = row0 + p * rpw;
        b[p] = (row < N && cl < nch) ? Bg[(int64_t)row * nch + cl] : CK::zero();
        t[p] = row < N ? thr[row] : 0;
    }
    for (int i = threadIdx.x; i < MS * nch; i += blockDim.x)
        As[i] = (i / nch < M) ? Ag[i] : CK::zero();
    __syncthreads();

    int acc[PASSES][MS];
#pragma unroll
    for (int p = 0; p < PASSES; ++p)
#pragma unroll
        for (int m = 0; m < MS; ++m)
            acc[p][m] = 0;
    for (int c = cl; c < nch; c += lpr) {
        chunk_t nxt[PASSES];
        const int cn = c + lpr;
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = row0 + p * rpw;
            nxt[p] = (row < N && cn < nch) ? Bg[(int64_t)row * nch + cn] : CK::zero();
        }
#pragma unroll
        for (int m = 0; m < MS; ++m) {
            const chunk_t a = As[m * nch + c];
#pragma unroll
            for (int p = 0; p < PASSES; ++p)
                acc[p][m] += CK::mism(a, b[p]);
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p)
            b[p] = nxt[p];
    }
    for (int off = lpr >> 1; off > 0; off >>= 1) {
#pragma unroll
        for (int p = 0; p < PASSES; ++p)
#pragma unroll
            for (int m = 0; m < MS; ++m)
                acc[p][m] += __shfl_xor(acc[p][m], off, kWave);
    }
    if (cl == 0) {
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = row0 + p * rpw;
#pragma unroll
            for (int m = 0; m < MS; ++m)
                decided[m][row - n_blk] = row < N && K_true - 2 * acc[p][m] >= t[p];
        }
    }
    __syncthreads();
    for (int m = wave; m < M; m += blockDim.x / kWave) {
        const uint64_t word = __ballot(lane < RB && decided[m][lane] != 0);
        if (lane != 0)
            continue;
        if (RB == 64) {
            out[(int64_t)m * gridDim.x + blockIdx.x] = word ^ (flip[blockIdx.x] & valid_cols_mask(blockIdx.x, N));
        } else {
            // quarter blockIdx.x % 4 of word blockIdx.x / 4 (little-endian: 16-bit piece j = bits 16 j ..)
            const uint64_t fl = (flip[blockIdx.x / 4] & valid_cols_mask(blockIdx.x / 4, N)) >> (16 * (blockIdx.x % 4));
            reinterpret_cast<uint16_t *>(out)[(int64_t)m * gridDim.x + blockIdx.x] = (uint16_t)(word ^ fl);
        }
    }
}

template <int MS, bool VEC16>
static int launch_gemv_bits2(const uint64_t *A, const uint64_t *B, const int32_t *thr, const uint64_t *flip,
                             uint64_t *out, int64_t M, int64_t N, int64_t K_true, int64_t row_words,
                             hipStream_t stream)
{
    const int nch = (int)(row_words / (VEC16 ? 2 : 1));
    int lpr = 1;
    while (lpr < kWave && lpr < nch)
        lpr <<= 1;
    // RB rows per block = waves * PASSES * (64 / lpr).  64 rows (up to 16 waves) when that still
    // gives every CU a block or the rows are too short to split further, else 16 (up to 4 waves);
    // the grid covers every 16-bit piece of the output words, also those beyond N (zeros)
    const int64_t Nw = ceil_div(N, 64);
    const int RB = (Nw >= 256 || lpr < 4) ? 64 : 16;
    const int total = RB * lpr / 64;
    const int maxw = RB == 64 ? 16 : 4;
    const int waves = total < maxw ? total : maxw;
    const int passes = total / waves;   // 1, 2 or 4
    const dim3 grid((unsigned)(RB == 64 ? Nw : 4 * Nw)), block((unsigned)(waves * kWave));
    const size_t lds = (size_t)MS * row_words * 8;
#define ESP_GEMV_BITS(P)                                                                                 \
    hipLaunchKernelGGL((bgemv_bits_kernel<MS, VEC16, P>), grid, block, lds, stream, A, B, thr, flip, out, \
                       (int)M, (int)N, (int)K_true, (int)row_words, lpr, RB)
    if (passes == 1)
        ESP_GEMV_BITS(1);
    else if (passes == 2)
        ESP_GEMV_BITS(2);
    else
        ESP_GEMV_BITS(4);
#undef ESP_GEMV_BITS
    return launch_status();
}

template <int MS>
static int launch_gemv_bits(const uint64_t *A, const uint64_t *B, const int32_t *thr, const uint64_t *flip,
                            uint64_t *out, int64_t M, int64_t N, int64_t K_true, int64_t row_words,
                            hipStream_t stream)
{
    const bool vec16 = (row_words % 2 == 0) && aligned(A, 16) && aligned(B, 16);
    return vec16 ? launch_gemv_bits2<MS, true>(A, B, thr, flip, out, M, N, K_true, row_words, stream)
                 : launch_gemv_bits2<MS, false>(A, B, thr, flip, out, M, N, K_true, row_words, stream);
}

int bgemm_launch(const uint64_t *A, const uint64_t *B, int32_t *C, int64_t M, int64_t N,
                 int64_t K_true, int64_t row_words, hipStream_t stream)
{
    if (M == 0)
        return ESP_OK;
    if (M >= (1ll << 31) || N >= (1ll << 31) || row_words >= (1ll << 29))
        return ESP_ESHAPE;
    if (M <= 1)
        return launch_gemv<1>(A, B, C, M, N, K_true, row_words, stream);
    if (M <= 2)
        return launch_gemv<2>(A, B, C, M, N, K_true, row_words, stream);
    if (M <= 4)
        return launch_gemv<4>(A, B, C, M, N, K_true, row_words, stream);
    if (M <= 8)
        return launch_gemv<8>(A, B, C, M, N, K_true, row_words, stream);
    // few columns (the 10 scores of the last layer): the same kernel with the operands swapped,
    // the few weight rows in LDS, the many activation rows streamed, C written transposed
    if (N <= 16 && (size_t)16 * row_words * 8 <= kGemvLdsBytes) {
        if (N <= 8)
            return launch_gemv<8>(B, A, C, N, M, K_true, row_words, stream, true);
        return launch_gemv<16>(B, A, C, N, M, K_true, row_words, stream, true);
    }
    TileOut o;
    o.C = C;
    return tile_matrix(A, B, o, M, N, K_true, row_words, stream);
}

int bgemm_bits_launch(const uint64_t *A, const uint64_t *B, const int32_t *thr, const uint64_t *flip,
                      uint64_t *out, int64_t M, int64_t N, int64_t K_true, int64_t row_words, int engine,
                      hipStream_t stream)
{
    if (M == 0)
        return ESP_OK;
    if (M >= (1ll << 31) || N >= (1ll << 31) || row_words >= (1ll << 29))
        return ESP_ESHAPE;
    // few rows: stream B once (as long as the packed rows of A fit in LDS), unless the caller
    // insists on the matrix cores
    const int ms = M <= 1 ? 1 : (M <= 2 ? 2 : (M <= 4 ? 4 : 8));
    if (engine != ESP_ENGINE_MFMA && M <= kGemvMaxM && (size_t)ms * row_words * 8 <= kGemvLdsBytes) {
        if (ms == 1)
            return launch_gemv_bits<1>(A, B, thr, flip, out, M, N, K_true, row_words, stream);
        if (ms == 2)
            return launch_gemv_bits<2>(A, B, thr, flip, out, M, N, K_true, row_words, stream);
        if (ms == 4)
            return launch_gemv_bits<4>(A, B, thr, flip, out, M, N, K_true, row_words, stream);
        return launch_gemv_bits<8>(A, B, thr, flip, out, M, N, K_true, row_words, stream);
    }
    if (resolve_engine(engine, M, N, K_true) == ESP_ENGINE_MFMA)
        return bgemm_mfma_launch(A, B, nullptr, thr, flip, out, M, N, K_true, row_words, stream);
    TileOut o;
    o.bits = out;
    o.thr = thr;
    o.flip = flip;
    return tile_matrix(A, B, o, M, N, K_true, row_words, stream);
}

bool bconv_implicit_ok(const uint64_t *in, const uint64_t *filt, int C)
{
    return C % 128 == 0 && aligned(in, 16) && aligned(filt, 16);
}

int bconv_implicit_launch(const uint64_t *in, const uint64_t *filt, int32_t *C_out, const int32_t *thr,
                          const uint64_t *flip, uint64_t *bits_out, int B, int H, int W, int C, int L2,
                          int kh, int kw, int stride, int pad, int H2, int W2, int pool_log2w, int engine,
                          hipStream_t stream)
{
    const int64_t M = (int64_t)B * H2 * W2;
    const int cdw = 2 * (C / 64);
    const int64_t row_dw = (int64_t)kh * kw * cdw;
    if (M >= (1ll << 31) || row_dw >= (1ll << 30) || (int64_t)B * H * W * cdw >= (1ll << 40))
        return ESP_ESHAPE;
    if (resolve_engine(engine, M, L2, (int64_t)kh * kw * C) == ESP_ENGINE_MFMA)
        return bconv_mfma_launch(in, filt, C_out, thr, flip, bits_out, B, H, W, C, L2, kh, kw, stride, pad,
                                 H2, W2, pool_log2w, stream);
    // stride-1 layers with enough whole-row tiles: filters resident in LDS, input streamed as patches
    if (bconv_patch_ok(in, filt, B, H, W, C, L2, kh, kw, stride, pad, H2, W2))
        return bconv_patch_launch(in, filt, C_out, thr, flip, bits_out, B, H, W, C, L2, kh, kw, stride, pad, H2, W2,
                                  pool_log2w, stream);
    const ConvA a = make_conv_a(in, B, H, W, C, kh, kw, stride, pad, H2, W2);
    TileOut o;
    o.C = C_out;
    o.bits = bits_out;
    o.thr = thr;
    o.flip = flip;
    o.pool_log2w = pool_log2w;
    if (bits_out && few_rows_ok(M, L2, row_dw, pool_log2w))
        return launch_few(a, reinterpret_cast<const uint32_t *>(filt), o, M, L2, (int64_t)kh * kw * C, row_dw,
                          stream);
    return launch_tile<ConvA, true>(a, reinterpret_cast<const uint32_t *>(filt), o, M, L2,
                                    (int64_t)kh * kw * C, row_dw, stream);
}

} // namespace esp

extern "C" int esp_bgemm(const uint64_t *A, const uint64_t *B, int32_t *C,
                         int64_t M, int64_t N, int64_t K, esp_stream stream)
{
    using namespace esp;
    if (M < 0 || N <= 0 || K <= 0)
        return ESP_EINVAL;
    if (K >= kMaxK)
        return ESP_ESHAPE;
    if (M == 0)
        return ESP_OK;
    if (!A || !B || !C)
        return ESP_EINVAL;
    if (!aligned(A, 8) || !aligned(B, 8) || !aligned(C, 4))
        return ESP_EALIGN;
    return bgemm_launch(A, B, C, M, N, K, ceil_div(K, 64), as_stream(stream));
}

extern "C" int esp_bgemm_bn_sign_pack(const uint64_t *A, const uint64_t *B, const int32_t *thr,
                                      const uint64_t *flip, uint64_t *out,
                                      int64_t M, int64_t N, int64_t K, int engine, esp_stream stream)
{
    using namespace esp;
    if (M < 0 || N <= 0 || K <= 0 || !engine_valid(engine))
        return ESP_EINVAL;
    if (K >= kMaxK)
        return ESP_ESHAPE;
    if (M == 0)
        return ESP_OK;
    if (!A || !B || !thr || !flip || !out)
        return ESP_EINVAL;
    if (!aligned(A, 8) || !aligned(B, 8) || !aligned(thr, 4) || !aligned(flip, 8) || !aligned(out, 8))
        return ESP_EALIGN;
    return bgemm_bits_launch(A, B, thr, flip, out, M, N, K, ceil_div(K, 64), engine, as_stream(stream));
}
