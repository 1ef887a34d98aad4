// Operand sources shared by the tiled binary-product kernels: 16-byte chunks of packed rows
// read either from a packed matrix or, for convolutions (arXiv 1705.07175, Sec. 5.2
// "Convolutional layers", Fig. 3), gathered straight from the packed NHWC input so that the
// lowered matrix never exists in memory.
#pragma once

#include "esp_internal.h"

namespace esp {

constexpr int kXcd = 8;       // XCDs (one L2 each); blocks are dealt to them round-robin
constexpr int kGroupM = 8;    // tile rows walked together so A and B slabs stay in one L2

// v with every bit cleared unless keep.  All loaders here are branch-free: they read from a
// clamped, always valid address and mask the result, so that a loader's independent loads are
// issued back to back instead of each inside its own branch.
__device__ __forceinline__ uint4 keep4(uint4 v, bool keep)
{
    const uint32_t m = keep ? 0xffffffffu : 0u;
    v.x &= m;
    v.y &= m;
    v.z &= m;
    v.w &= m;
    return v;
}

// 16 bytes of row p from dword kd on, zeros beyond row_dw, without a branch (row_dw >= 4 with
// VEC16, row_dw >= 2 and even otherwise).
template <bool VEC16>
__device__ __forceinline__ uint4 load_chunk_nb(const uint32_t *__restrict__ p, int kd, int row_dw)
{
    if (VEC16)
        return keep4(*reinterpret_cast<const uint4 *>(p + min(kd, row_dw - 4)), kd < row_dw);
    const uint2 lo = *reinterpret_cast<const uint2 *>(p + min(kd, row_dw - 2));
    const uint2 hi = *reinterpret_cast<const uint2 *>(p + min(kd + 2, row_dw - 2));
    const uint32_t m0 = kd < row_dw ? 0xffffffffu : 0u, m1 = kd + 2 < row_dw ? 0xffffffffu : 0u;
    return make_uint4(lo.x & m0, lo.y & m0, hi.x & m1, hi.y & m1);
}

// load_chunk_nb without the final mask where a single mask covers the chunk (VEC16: the caller
// applies keep4(v, kd < row_dw) when it uses the data, so that nothing waits for the load at
// the point of issue); the 8-byte path masks its halves at once.
template <bool VEC16>
__device__ __forceinline__ uint4 load_chunk_raw(const uint32_t *__restrict__ p, int kd, int row_dw)
{
    if (VEC16)
        return *reinterpret_cast<const uint4 *>(p + min(kd, row_dw - 4));
    return load_chunk_nb<false>(p, kd, row_dw);
}

// ---- A operand: rows of a packed matrix ------------------------------------------
template <bool VEC16>
struct MatrixA {
    static constexpr bool kGathered = false;   // a row is one contiguous run of memory
    const uint32_t *base;
    int rows;    // M
    int row_dw;  // dwords per row
    struct Row { const uint32_t *p; };
    struct Step {};
    __device__ __forceinline__ Step step(int /*kd*/) const { return Step{}; }
    // rows beyond the matrix read the last row (their results are never stored)
    __device__ __forceinline__ Row row_nb(int r) const { return Row{base + (int64_t)min(r, rows - 1) * row_dw}; }
    __device__ __forceinline__ uint4 fetch_nb(const Row &r, const Step &, int kd) const
    {
        return load_chunk_nb<VEC16>(r.p, kd, row_dw);
    }
    // the same in two parts, so that the mask can wait until the data is used: fetch_raw reads
    // the clamped address, keep() says whether the chunk counts (keep4(fetch_raw, keep) ==
    // fetch_nb)
    __device__ __forceinline__ uint4 fetch_raw(const Row &r, const Step &, int kd) const
    {
        return load_chunk_raw<VEC16>(r.p, kd, row_dw);
    }
    __device__ __forceinline__ bool keep(const Row &, const Step &, int kd) const { return kd < row_dw; }
};

// ---- A operand: the lowered matrix of a convolution, gathered on the fly ----------
// Row r = (b*H2 + m)*W2 + n is the sliding volume of output pixel (b, m, n); dword kd of
// that row is dword kd % cdw of input pixel (m*s - p + dy, n*s - p + dx) with
// tap = kd / cdw = dy*kw + dx; pixels outside the image read as zero words (= -1).
// Needs cdw % 4 == 0 (C a multiple of 128) so that a 16-byte chunk never straddles taps.
struct ConvA {
    static constexpr bool kGathered = true;    // a row is kh * kw runs found by index arithmetic
    const uint32_t *in;
    int rows;    // B*H2*W2
    int row_dw;  // kh*kw*cdw
    int H, W, cdw, stride, pad;
    FastDiv d_w2, d_h2, d_cdw, d_kw;
    struct Row { int64_t img; int y0, x0; };
    // rows beyond M read the last row (their results are never stored)
    __device__ __forceinline__ Row row_nb(int r0) const
    {
        const int r = min(r0, rows - 1);
        const uint32_t bm = fd_div((uint32_t)r, d_w2);
        const uint32_t n = (uint32_t)r - bm * d_w2.div;
        const uint32_t b = fd_div(bm, d_h2);
        const uint32_t m = bm - b * d_h2.div;
        return Row{(int64_t)b * H * W, (int)(m * stride) - pad, (int)(n * stride) - pad};
    }
    struct Step { int dy, dx, c; };
    __device__ __forceinline__ Step step(int kd) const
    {
        const uint32_t tap = fd_div((uint32_t)kd, d_cdw);
        const uint32_t dy = fd_div(tap, d_kw);
        return Step{(int)dy, (int)(tap - dy * d_kw.div), (int)((uint32_t)kd - tap * d_cdw.div)};
    }
    // the pixel is clamped into the image, the border and the K tail are masked
    __device__ __forceinline__ uint4 fetch_nb(const Row &r, const Step &s, int kd) const
    {
        const int y = r.y0 + s.dy, x = r.x0 + s.dx;
        const bool inside = kd < row_dw && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)W;
        const int yc = min(max(y, 0), H - 1), xc = min(max(x, 0), W - 1);
        return keep4(*reinterpret_cast<const uint4 *>(in + (r.img + (int64_t)yc * W + xc) * cdw + s.c), inside);
    }
    __device__ __forceinline__ uint4 fetch_raw(const Row &r, const Step &s, int kd) const
    {
        const int yc = min(max(r.y0 + s.dy, 0), H - 1), xc = min(max(r.x0 + s.dx, 0), W - 1);
        return *reinterpret_cast<const uint4 *>(in + (r.img + (int64_t)yc * W + xc) * cdw + s.c);
    }
    __device__ __forceinline__ bool keep(const Row &r, const Step &s, int kd) const
    {
        const int y = r.y0 + s.dy, x = r.x0 + s.dx;
        return kd < row_dw && (unsigned)y < (unsigned)H && (unsigned)x < (unsigned)W;
    }
};

// Host side: describe the implicit lowered matrix of a convolution (C a multiple of 128).
inline ConvA make_conv_a(const uint64_t *in, int B, int H, int W, int C, int kh, int kw, int stride,
                         int pad, int H2, int W2)
{
    ConvA a;
    a.in = reinterpret_cast<const uint32_t *>(in);
    a.rows = B * H2 * W2;
    a.cdw = 2 * (C / 64);
    a.row_dw = kh * kw * a.cdw;
    a.H = H;
    a.W = W;
    a.stride = stride;
    a.pad = pad;
    a.d_w2 = make_fastdiv((uint32_t)W2);
    a.d_h2 = make_fastdiv((uint32_t)H2);
    a.d_cdw = make_fastdiv((uint32_t)a.cdw);
    a.d_kw = make_fastdiv((uint32_t)kw);
    return a;
}

// Block id -> (tile row, tile column).  Consecutive block ids land on different XCDs, so
// every XCD gets a contiguous range of tiles, walked in groups of kGroupM tile rows.
// Returns false for the padding blocks beyond the last tile.
__device__ __forceinline__ bool block_to_tile(int tiles_m, int tiles_n, int tiles_per_xcd, int *tm, int *tn)
{
    const int pid = blockIdx.x;
    const int tile = (pid % kXcd) * tiles_per_xcd + pid / kXcd;
    if (tile >= tiles_m * tiles_n)
        return false;
    const int group_size = kGroupM * tiles_n;
    const int first_m = (tile / group_size) * kGroupM;
    const int gm = min(tiles_m - first_m, kGroupM);
    const int in_group = tile % group_size;
    *tm = first_m + in_group % gm;
    *tn = in_group / gm;
    return true;
}

// Fused 2x2 / stride-2 max-pool behind the sign (Sec. 6.3: pooling acts on +-1 activations,
// so the maximum is the OR of the sign bits).  wt holds the BM x WPT packed words of a block
// tile whose BM rows are whole pairs of image rows (BM a multiple of 2 * W2, W2 = 1 << log2w,
// tile origin m0 a multiple of BM): pooled row m0/4 + pp ORs local rows
// 2*pl*W2 + 2*pn + {0, 1, W2, W2 + 1} with pl = pp / (W2/2), pn = pp % (W2/2).
// M is a multiple of 2 * W2, so a pooled row is valid exactly when it is below M / 4.
template <int BM, int WPT, int NT>
__device__ __forceinline__ void pool_tile_store(const uint64_t *wt, uint64_t *__restrict__ out, int m0,
                                                int n0, int M, int Nw, int log2w, int tid)
{
    const int W2 = 1 << log2w;
    for (int t = tid; t < (BM / 4) * WPT; t += NT) {
        const int wl = t % WPT, pp = t / WPT;
        const int pl = pp >> (log2w - 1), pn = pp & ((W2 >> 1) - 1);
        const int base = ((2 * pl) << log2w) + 2 * pn;
        const uint64_t v = wt[base * WPT + wl] | wt[(base + 1) * WPT + wl] | wt[(base + W2) * WPT + wl] |
                           wt[(base + W2 + 1) * WPT + wl];
        const int prow = (m0 >> 2) + pp;
        const int w = (n0 >> 6) + wl;
        if (prow < (M >> 2) && w < Nw)
            out[(int64_t)prow * Nw + w] = v;
    }
}

} // namespace esp
