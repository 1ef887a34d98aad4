// Internal helpers shared by the kernels of the gfx950 binary-network library.
// Nothing here is part of the C ABI (see include/espresso_hip.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "espresso_hip.h"

namespace esp {

constexpr int kWave = 64;            // gfx950 wavefront size
constexpr int64_t kMaxK = 1ll << 30; // |dot| <= K must fit int32 with headroom

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline hipStream_t as_stream(esp_stream s) { return reinterpret_cast<hipStream_t>(s); }

// Status of the launch that was just enqueued.
inline int launch_status() { return hipGetLastError() == hipSuccess ? ESP_OK : ESP_ELAUNCH; }

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

inline bool engine_valid(int e) { return e == ESP_ENGINE_XOR_POPCOUNT || e == ESP_ENGINE_MFMA || e == ESP_ENGINE_AUTO; }

// ESP_ENGINE_AUTO -> a concrete engine for an M x N product of length K.  Measured break-even
// of the two engines on the networks' layers: the matrix cores win from 32 of their 256 x 128
// tiles on, provided a tile's 256 rows exist (a dense layer at batch 128 is better off on the
// vector ALUs, at batch 256 on the matrix cores).
inline int resolve_engine(int e, int64_t M, int64_t N, int64_t K)
{
    if (e != ESP_ENGINE_AUTO)
        return e;
    const int64_t tiles = ceil_div(M, 256) * ceil_div(N, 128);
    return (tiles >= 32 && M >= 256 && K < (1ll << 24)) ? ESP_ENGINE_MFMA : ESP_ENGINE_XOR_POPCOUNT;
}

// Division of a 32-bit unsigned value by a run-time constant, done as a
// multiply-high and a shift (round-up method, exact for n < 2^31).
struct FastDiv {
    uint32_t mul;
    uint32_t shift;
    uint32_t div;
};

inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.div = d;
    if (d == 1) {
        f.mul = 0;
        f.shift = 0;
        return f;
    }
    uint32_t l = 0;
    while ((1ull << l) < d)
        ++l; // l = ceil(log2 d)
    const uint64_t m = ((1ull << (31 + l)) + d - 1) / d;
    f.mul = static_cast<uint32_t>(m);
    f.shift = l - 1;
    return f;
}

__device__ __forceinline__ uint32_t fd_div(uint32_t n, const FastDiv f)
{
    // mul = ceil(2^(31+l) / d) with l = ceil(log2 d): (n * mul) >> (31 + l) == n / d for n < 2^31.
    return f.div == 1 ? n : (__umulhi(n, f.mul) >> f.shift);
}

// Bits of 64-column word w that belong to real columns (n < N).  A caller's flip word may carry
// set bits beyond N; they must not reach the packed output, whose tail bits are zero by the
// packing convention (the next product relies on that).
__host__ __device__ __forceinline__ uint64_t valid_cols_mask(int w, int N)
{
    const int left = N - w * 64;
    return left >= 64 ? ~0ull : (left <= 0 ? 0ull : ((1ull << left) - 1ull));
}

// Consecutive block ids run on different XCDs (eight, each with its own L2).  For a grid that is a
// multiple of 8 blocks this gives block b the logical index that cuts the grid into eight
// contiguous ranges, one per XCD, so that neighbouring pieces of work share an L2.
__device__ __forceinline__ uint32_t xcd_contiguous_block()
{
    const uint32_t per_xcd = gridDim.x / 8;
    return (gridDim.x % 8 == 0) ? (blockIdx.x % 8) * per_xcd + blockIdx.x / 8 : blockIdx.x;
}

// Number of blocks for a grid-stride kernel.  Measured on MI355X, streaming kernels reach
// their best HBM bandwidth when the grid covers the whole array with one item per thread
// (blocks are dispatched in order, so the blocks in flight sweep memory as one front);
// a few thousand blocks looping with a large stride lose 20-30 %.  Hence the high cap:
// the loops in the kernels only matter for arrays beyond it.
inline unsigned grid_for(int64_t work_items, int per_block, int64_t max_blocks = 1ll << 30)
{
    int64_t b = ceil_div(work_items, per_block);
    if (b < 1)
        b = 1;
    if (b > max_blocks)
        b = max_blocks;
    return static_cast<unsigned>(b);
}

// bgemm on raw word rows whose stored width (row pitch in uint64 words) is
// given separately from the true bit length K: the lowered matrix of a
// convolution pads every tap to whole words, so its pitch is not ceil(K/64).
int bgemm_launch(const uint64_t *A, const uint64_t *B, int32_t *C, int64_t M, int64_t N,
                 int64_t K_true, int64_t row_words, hipStream_t stream);

// Same product with the folded batch-norm threshold + sign applied in the epilogue:
// out [M][ceil(N/64)] packed bits instead of int32 dots.  engine: esp_engine.
int bgemm_bits_launch(const uint64_t *A, const uint64_t *B, const int32_t *thr, const uint64_t *flip,
                      uint64_t *out, int64_t M, int64_t N, int64_t K_true, int64_t row_words, int engine,
                      hipStream_t stream);

// Matrix-core version of the product; exactly one of C (int32 dots) and bits (+ thr, flip).
int bgemm_mfma_launch(const uint64_t *A, const uint64_t *B, int32_t *C, const int32_t *thr,
                      const uint64_t *flip, uint64_t *bits, int64_t M, int64_t N, int64_t K_true,
                      int64_t row_words, hipStream_t stream);

// Dense layer on 8-bit inputs given as bit-planes [rows][8][row_words] (Eq. 3), on the matrix
// cores, the planes combined in the epilogue: y int32 [rows][N] and / or bits (+ thr, flip).
int bitplane_dense_mfma_launch(const uint64_t *planes, const uint64_t *W, const int32_t *wsum, int32_t *y,
                               const int32_t *thr, const uint64_t *flip, uint64_t *bits, int64_t rows, int64_t N,
                               int64_t K_true, int64_t row_words, hipStream_t stream);

// Convolution without a lowered matrix: the tile loader gathers the sliding volumes from
// the packed NHWC input.  Usable when C is a multiple of 128 and the buffers are 16-byte
// aligned.  Exactly one of C_out (int32 [B][H2][W2][L2]) and bits_out (+ thr, flip) is set.
// pool_log2w != 0 (bits_out only): a 2x2 / stride-2 max-pool is applied to the sign bits in
// the epilogue and bits_out is [B][H2/2][W2/2][ceil(L2/64)]; needs H2 even and
// W2 == 1 << pool_log2w with 2 <= W2 <= 64.
bool bconv_implicit_ok(const uint64_t *in, const uint64_t *filt, int C);
int bconv_implicit_launch(const uint64_t *in, const uint64_t *filt, int32_t *C_out, const int32_t *thr,
                          const uint64_t *flip, uint64_t *bits_out, int B, int H, int W, int C, int L2,
                          int kh, int kw, int stride, int pad, int H2, int W2, int pool_log2w, int engine,
                          hipStream_t stream);
// The same for stride-1 convolutions whose block tiles are whole image rows: filters resident in
// LDS, the input streamed as patches (bconv_patch.hip).  bconv_patch_ok says whether a shape
// qualifies; XOR-popcount engine only.
bool bconv_patch_ok(const uint64_t *in, const uint64_t *filt, int B, int H, int W, int C, int L2, int kh, int kw,
                    int stride, int pad, int H2, int W2);
int bconv_patch_launch(const uint64_t *in, const uint64_t *filt, int32_t *C_out, const int32_t *thr,
                       const uint64_t *flip, uint64_t *bits_out, int B, int H, int W, int C, int L2, int kh, int kw,
                       int stride, int pad, int H2, int W2, int pool_log2w, hipStream_t stream);
int bconv_mfma_launch(const uint64_t *in, const uint64_t *filt, int32_t *C_out, const int32_t *thr,
                      const uint64_t *flip, uint64_t *bits_out, int B, int H, int W, int C, int L2,
                      int kh, int kw, int stride, int pad, int H2, int W2, int pool_log2w,
                      hipStream_t stream);

} // namespace esp
