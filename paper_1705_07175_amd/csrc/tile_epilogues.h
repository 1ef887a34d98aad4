// Pieces shared by the tiled binary-product kernels (arXiv 1705.07175, Sec. 4.2, Eq. 2): the
// inner xor + popcount step, and the two epilogues -- int32 dot products, or the folded
// batch-norm threshold + sign packed into words (the bit-packing sign activation of Sec. 6.3).
#pragma once

#include "esp_internal.h"

namespace esp {

// ---- epilogue: int32 dot products ---------------------------------------------------
struct StoreDots {
    int32_t *C;
    int vec_store;
    // a lane owns, per row, TN/4 runs of four consecutive columns
    template <int TN, int TX>
    __device__ __forceinline__ void row(int r, int N, int K_true, int n0, int tx, const int (&acc)[TN]) const
    {
        int32_t *crow = C + (int64_t)r * N;
#pragma unroll
        for (int jg = 0; jg < TN / 4; ++jg) {
            const int col = n0 + jg * 4 * TX + tx * 4;
            int4 v;
            v.x = K_true - 2 * acc[jg * 4 + 0];
            v.y = K_true - 2 * acc[jg * 4 + 1];
            v.z = K_true - 2 * acc[jg * 4 + 2];
            v.w = K_true - 2 * acc[jg * 4 + 3];
            if (vec_store && col + 3 < N) {
                *reinterpret_cast<int4 *>(crow + col) = v;
            } else {
                if (col + 0 < N) crow[col + 0] = v.x;
                if (col + 1 < N) crow[col + 1] = v.y;
                if (col + 2 < N) crow[col + 2] = v.z;
                if (col + 3 < N) crow[col + 3] = v.w;
            }
        }
    }
};

// Value of `v` held by lane (lane ^ S) of the same 16-lane row.
template <int S>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v)
{
    if (S == 1)
        return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1 /* quad_perm [1,0,3,2] */, 0xf, 0xf, true);
    if (S == 2)
        return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E /* quad_perm [2,3,0,1] */, 0xf, 0xf, true);
    if (S == 4)
        return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x101F /* lane ^ 4 */);
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128 /* row_ror:8 == lane ^ 8 */, 0xf, 0xf, true);
}

// One butterfly step of a 16 x 16 nibble transpose across the 16 lanes of a row, on a
// register holding 8 nibbles: lanes whose index has bit S clear keep the nibbles at
// positions with bit S clear and receive, into the other positions, the partner's kept
// nibbles moved up by S positions; lanes with bit S set do the mirror image.
template <int S>
__device__ __forceinline__ uint32_t nibble_swap(uint32_t own, bool lane_bit)
{
    constexpr uint32_t kHigh = S == 1 ? 0xF0F0F0F0u : (S == 2 ? 0xFF00FF00u : 0xFFFF0000u);
    const uint32_t p = lane_xor<S>(own);
    const uint32_t moved = __builtin_amdgcn_alignbit(p, p, lane_bit ? 4 * S : 32 - 4 * S);
    const uint32_t keep = lane_bit ? kHigh : ~kHigh;
    return (keep & own) | (~keep & moved);
}

// ---- epilogue: folded batch-norm threshold + sign, packed ---------------------------
// bit n of row r = (dot >= thr[n]) XOR flipbit(n).  The 16 lanes tx = 0..15 that share the
// rows ty + TY*i each hold, per row and 64-column word, four consecutive bits (a nibble).
// Instead of reducing every word over the 16 lanes, the nibbles are transposed across the
// lanes (4 butterfly steps on two registers), after which lane tx holds one complete word.
// Requires TX == 16 and a tile origin n0 that is a multiple of 64; all 64 lanes must call.
struct LaneWord {
    int rl, wl;             // row and 64-column word inside the block tile
    bool have;              // this lane holds a word
    uint32_t lo, hi;
};

// x = 2 x + (a <= lim): the comparison's carry shifts the decision in from the right -- two
// vector instructions per output bit (compare, add-with-carry) instead of compare, select, or.
// Decisions are therefore fed from the highest bit of the register down to the lowest.
__device__ __forceinline__ void shift_in_le(uint32_t &x, int a, int lim)
{
    asm volatile("v_cmp_le_i32 vcc, %1, %2\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(x) : "v"(a), "v"(lim) : "vcc");
}

struct StoreSignBits {
    uint64_t *out;          // [M][Nw], or [M/4][Nw] behind a fused 2x2 max-pool
    const int32_t *thr;     // [N]
    const uint64_t *flip;   // [Nw]
    int Nw;
    int N;                  // columns; flip bits beyond them are ignored
    int pool_log2w;         // 0: no pooling; else log2 of the output width W2 of the convolution

    // mismatch-count threshold: dot = K - 2a >= thr  <=>  a <= floor((K - thr) / 2)
    __device__ __forceinline__ int mismatch_limit(int col, int N, int K_true) const
    {
        if (col >= N)
            return -1;                                    // tail bits stay 0
        const int t = min(max(thr[col], -K_true), K_true + 1);
        return (K_true - t) >> 1;
    }

    // final bits of a lane's word (0 beyond the last word of the row)
    __device__ __forceinline__ uint64_t finish(const LaneWord &lw, int w) const
    {
        return (lw.have && w < Nw) ? ((((uint64_t)lw.hi << 32) | lw.lo) ^ (flip[w] & valid_cols_mask(w, N))) : 0ull;
    }

    // 8 x 8 counters per lane: slots q = jg*8 + i, lo register = word jg 0, hi = word jg 1
    template <int TY>
    __device__ __forceinline__ LaneWord tile(const int (&acc)[8][8], const int (&lim)[8], int tx, int ty) const
    {
        uint32_t lo = 0, hi = 0;     // bit 4 i + c of lo / hi: row i, column c / 4 + c
#pragma unroll
        for (int i = 7; i >= 0; --i)
#pragma unroll
            for (int c = 3; c >= 0; --c) {
                shift_in_le(lo, acc[i][c], lim[c]);
                shift_in_le(hi, acc[i][4 + c], lim[4 + c]);
            }
        lo = nibble_swap<1>(lo, tx & 1);
        hi = nibble_swap<1>(hi, tx & 1);
        lo = nibble_swap<2>(lo, tx & 2);
        hi = nibble_swap<2>(hi, tx & 2);
        lo = nibble_swap<4>(lo, tx & 4);
        hi = nibble_swap<4>(hi, tx & 4);
        // step 8 moves whole registers: lanes 0-7 take the partner's lo as their hi, lanes
        // 8-15 take the partner's hi as their lo
        const bool up = tx & 8;
        const uint32_t got = lane_xor<8>(up ? lo : hi);
        lo = up ? got : lo;
        hi = up ? hi : got;
        // lane tx now holds the word of slot q = tx: row ty + TY*(tx % 8), word tx / 8
        return LaneWord{ty + TY * (tx & 7), tx >> 3, true, lo, hi};
    }

    // 8 x 4 counters per lane: the tile is one word wide, a lane's register holds one nibble
    // for each of its 8 rows
    template <int TY>
    __device__ __forceinline__ LaneWord tile_8x4(const int (&acc)[8][4], const int (&lim)[4], int tx, int ty) const
    {
        uint32_t x = 0;              // bit 4 i + c: row i, column c
#pragma unroll
        for (int i = 7; i >= 0; --i)
#pragma unroll
            for (int c = 3; c >= 0; --c)
                shift_in_le(x, acc[i][c], lim[c]);
        x = nibble_swap<1>(x, tx & 1);
        x = nibble_swap<2>(x, tx & 2);
        x = nibble_swap<4>(x, tx & 4);
        // lane tx now holds, of row ty + TY*(tx % 8), the 32 bits that belong to the 8 lanes of
        // its half: lanes 0-7 the low half of the word, lanes 8-15 the high half
        const uint32_t other = lane_xor<8>(x);
        return LaneWord{ty + TY * (tx & 7), 0, tx < 8, x, other};
    }

    // TM x 4 counters per lane (TM = 1, 2 or 4): one word per row i < TM
    template <int TY, int TM>
    __device__ __forceinline__ LaneWord tile(const int (&acc)[TM][4], const int (&lim)[4], int tx, int ty) const
    {
        static_assert(TM <= 4, "rows per lane");
        uint32_t x = 0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                x |= acc[i][c] <= lim[c] ? 0x10001u << (4 * i + c) : 0u;   // kept 16-bit periodic
        x = nibble_swap<1>(x, tx & 1);
        x = nibble_swap<2>(x, tx & 2);
        // the quad tx/4 now holds, in lane tx, its 16 bits of the word of row i = tx % 4
        const uint32_t piece = (x & 0xFFFFu) << (16 * ((tx >> 2) & 1));
        uint32_t lo = (tx & 8) ? 0u : piece;
        uint32_t hi = (tx & 8) ? piece : 0u;
        lo |= lane_xor<4>(lo);
        hi |= lane_xor<4>(hi);
        lo |= lane_xor<8>(lo);
        hi |= lane_xor<8>(hi);
        return LaneWord{ty + TY * tx, 0, tx < TM, lo, hi};
    }
};

// acc += popcount(a XOR b) over the four dwords of two 16-byte chunks: the inner step of Eq. 2.
// Written out as instructions because their order decides the rate on gfx950: v_xor_b32 issues
// in half the time of v_bcnt_u32_b32, but two waves that share a SIMD only overlap that way when
// a scalar instruction separates the pairs (measured on registers only, two waves per SIMD:
// xor, bcnt back to back 1.24 Pbop/s; one s_nop per pair 1.63; two, or one per two pairs, 1.2).
// The compiler places one more s_nop between consecutive asm statements, which is the
// separator of the fourth pair.
__device__ __forceinline__ void xor_popc_acc4(int &acc, const uint4 &a, const uint4 &b)
{
    uint32_t t;
    asm volatile("v_xor_b32 %0, %2, %6\n\tv_bcnt_u32_b32 %1, %0, %1\n\ts_nop 0\n\t"
                 "v_xor_b32 %0, %3, %7\n\tv_bcnt_u32_b32 %1, %0, %1\n\ts_nop 0\n\t"
                 "v_xor_b32 %0, %4, %8\n\tv_bcnt_u32_b32 %1, %0, %1\n\ts_nop 0\n\t"
                 "v_xor_b32 %0, %5, %9\n\tv_bcnt_u32_b32 %1, %0, %1"
                 : "=&v"(t), "+v"(acc)
                 : "v"(a.x), "v"(a.y), "v"(a.z), "v"(a.w), "v"(b.x), "v"(b.y), "v"(b.z), "v"(b.w));
}

// The same for the first k-group of a tile: acc = popcount(a XOR b), so that the counters need
// no zeroing (one vector instruction per counter and tile).
__device__ __forceinline__ void xor_popc_set4(int &acc, const uint4 &a, const uint4 &b)
{
    uint32_t t;
    asm volatile("v_xor_b32 %0, %2, %6\n\tv_bcnt_u32_b32 %1, %0, 0\n\ts_nop 0\n\t"
                 "v_xor_b32 %0, %3, %7\n\tv_bcnt_u32_b32 %1, %0, %1\n\ts_nop 0\n\t"
                 "v_xor_b32 %0, %4, %8\n\tv_bcnt_u32_b32 %1, %0, %1\n\ts_nop 0\n\t"
                 "v_xor_b32 %0, %5, %9\n\tv_bcnt_u32_b32 %1, %0, %1"
                 : "=&v"(t), "=&v"(acc)
                 : "v"(a.x), "v"(a.y), "v"(a.z), "v"(a.w), "v"(b.x), "v"(b.y), "v"(b.z), "v"(b.w));
}

} // namespace esp
