// Binary convolution with the filters resident in LDS and the input streamed as image
// patches (arXiv 1705.07175, Sec. 5.2 "Convolutional layers", Fig. 3; product of Eq. 2).
//
// The lowered matrix of Fig. 3 repeats every input pixel kh * kw times.  The general tile
// kernel gathers those copies into LDS stage by stage; here a block tile of 128 consecutive
// output pixels (whole image rows) keeps its input PATCH -- the rows it covers plus the
// (kh - 1) x (kw - 1) halo, border pixels as zero words (= -1) -- in LDS once, and a lane
// reads the operand of output pixel x at tap (dy, dx) from patch pixel (y + dy, x + dx).
// A lane owns 8 consecutive pixels of one image row, so its eight operands of a k-group are
// one LDS address plus immediates, and that address advances by one 16-byte chunk per
// k-group (by the row pitch when dy changes).  A 3 x 3 layer's K is short (1152 - 4608 bits):
// the block's 64 or 128 filters stay in LDS for all of it, and the block walks several row tiles,
// fetching the next patch (1 - 4 chunks per thread) while it counts the current one, so that
// after the first tile nothing waits for memory.  Per tile: one barrier.
// With 128 filters per block a lane keeps 8 x 8 counters: every operand read from LDS then
// serves twice as many xor + popcount pairs (12 reads per 128 pairs become 16 per 256), which
// is what two waves per SIMD need to keep the vector ALUs fed (conv2 of the Sec. 6.3 network at
// batch 256: 60.9 -> 57.4 us; conv4: 58.9 -> 56.5).  It is taken whenever the layer has a
// multiple of 128 filters, their slab fits LDS beside the patches (up to 256 channels for a
// 3 x 3 layer) and the grid still gets a tile per block.
//
// Used for stride-1 convolutions on 128, 256 or 512 channels whose output width is a power
// of two between 8 and 128 (the layers of the Sec. 6.3 network); everything else takes the
// gathering tile kernel.  Same results: int32 dots, or threshold + sign (+ 2x2 OR pool).
#include <type_traits>

#include "esp_internal.h"
#include "tile_sources.h"
#include "tile_epilogues.h"

namespace esp {

// Block tile: 128 output pixels x 64 or 128 filters; a lane keeps 8 x TN counters, TN = 4 or 8
// (its columns are TN / 4 runs of four, 64 apart, as in the tile kernel).
constexpr int kPBM = 128;
constexpr int kPTM = 8;
constexpr int kPTX = 16, kPTY = kPBM / kPTM, kPNT = kPTX * kPTY;   // 16 x 16 lanes
constexpr int kPatchMaxChunksPerThread = 4;   // a patch is at most 4 * 256 chunks of 16 bytes
constexpr int kPatchMaxKG = 36;            // k-groups (128 bits each) of a filter: 3 x 3 x 512 channels
constexpr int kPatchSlots = 2 * 256;       // blocks of a launch: two per compute unit
constexpr size_t kPatchMaxLdsWide = 144 * 1024;   // a block of two halves has the CU to itself

struct PatchGeom {
    const uint32_t *in;      // packed NHWC input
    int B, H, W, pad;
    int M;                   // output pixels B * H2 * W2
    int log2w;               // W2 = 1 << log2w
    int log2pix;             // log2 of the output pixels of one image inside a tile
    int nimg;                // images per tile (1 when a tile lies inside one image)
    int rows_img;            // output rows of one image inside a tile
    int prow, pcol;          // patch rows per image, pixels per patch row
    int pitch;               // chunks per patch row in LDS
    int patch_chunks;        // chunks to fetch per tile: nimg * prow * pcol * CPP
    int patch_lds_chunks;    // nimg * prow * pitch
    int kwc;                 // k-groups per filter row: kw * CPP
    int KG;                  // k-groups per filter: kh * kw * CPP
    int cdw;                 // dwords per input pixel
    FastDiv d_pcol, d_prow, d_tpi;         // divisions by pcol, prow, tiles per image
};

template <int CPP, int PCH, bool BITS, int TN, int NH>
__global__ __launch_bounds__(kPNT * NH, NH == 2 ? 1 : (TN == 4 ? 3 : 2))
void bconv_patch_kernel(const PatchGeom g, const uint32_t *__restrict__ filt, const StoreDots dots,
                        const StoreSignBits bits, int N, int K_true, int tiles_m, int tiles_n, int G)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    constexpr int kPTN = TN, kPBN = kPTX * TN, kPWords = kPBN / 64;
    constexpr int kPatchBPitch = kPBN + 1;     // chunks per k-group of the filter slab (+1: bank skew)
    // NH = 2: the block is two halves of 256 threads that share the filter slab; each half walks
    // its own row tiles (tile 2 p + half of the block's pair p) with its own patch buffers.
    const int half = NH == 1 ? 0 : __builtin_amdgcn_readfirstlane(threadIdx.x / kPNT);
    uint4 *Bs = reinterpret_cast<uint4 *>(smem_raw);                     // [KG][kPatchBPitch]
    uint4 *P0 = Bs + g.KG * kPatchBPitch + half * 2 * g.patch_lds_chunks;   // two patch buffers per half
    uint4 *P1 = P0 + g.patch_lds_chunks;
    uint64_t *wt_all = reinterpret_cast<uint64_t *>(Bs + g.KG * kPatchBPitch + NH * 2 * g.patch_lds_chunks);
    uint64_t *wt = wt_all + half * kPBM * kPWords;                       // [kPBM][kPWords] words for the pooled epilogue
    uint64_t *flip_s = wt_all + NH * kPBM * kPWords;                     // the block's flip words (two slots)
    int *lim_s = reinterpret_cast<int *>(flip_s + 2);                    // [kPBN] mismatch limits (16-byte aligned)

    const int tid = threadIdx.x % kPNT;          // index inside the half
    const int tx = tid % kPTX;
    const int tyl = tid / kPTX;
    // the four lane rows of a wave take pixel groups 32 tile rows apart, so that their operand
    // reads fall into different LDS banks
    const int ty = (tyl % 4) * 4 + tyl / 4;
    const int tn = blockIdx.x % tiles_n;
    const int first = blockIdx.x / tiles_n;      // this block walks row tiles (pairs) first, first + G, ...
    const int n0 = tn * kPBN;
    const int walks = (tiles_m + NH - 1) / NH;   // row tiles, or pairs of them
    if (first >= walks)
        return;

    // ---- patch fetch: chunk q of the patch <-> (image, patch row, patch pixel, part) -----
    // What does not depend on the tile is worked out once per block when a thread has one or two
    // chunks (the Sec. 6.3 layers): the chunk's offset from the tile's first input pixel, the
    // range of tile rows for which its image row exists, its image within the tile.  Threads with
    // four chunks decode on every fetch instead (the registers are needed elsewhere).
    constexpr bool kKeepDecode = PCH <= 2;
    uint32_t p_rel[kKeepDecode ? PCH : 1], p_ymin[kKeepDecode ? PCH : 1], p_il[kKeepDecode ? PCH : 1];
    uint32_t p_dst[kKeepDecode ? PCH : 1];       // where the chunk goes in a patch buffer
    if constexpr (kKeepDecode) {
#pragma unroll
        for (int i = 0; i < PCH; ++i) {
            const uint32_t q = tid + i * kPNT;
            const uint32_t qq = min(q, (uint32_t)g.patch_chunks - 1);
            const uint32_t pix = qq / CPP, part = qq % CPP;
            const uint32_t t = fd_div(pix, g.d_pcol), px = pix - t * g.pcol;
            const uint32_t il = fd_div(t, g.d_prow), py = t - il * g.prow;
            const int x = (int)px - g.pad;
            const bool x_ok = q < (uint32_t)g.patch_chunks && (unsigned)x < (unsigned)g.W;
            // offset of input pixel (il, py - pad, px - pad) from pixel (0, 0, 0), in dwords, modulo 2^32
            p_rel[i] = ((il * g.H + py - g.pad) * g.W + x) * g.cdw + part * 4;
            p_ymin[i] = (uint32_t)(g.pad - (int)py);     // the chunk's image row is y0 - p_ymin
            p_il[i] = x_ok ? il : 0x7fffffffu;           // never below B - b0: such a chunk never counts
            p_dst[i] = t * g.pitch + px * CPP + part;
        }
    }
    uint4 pp[PCH];                                // PCH * 256 chunks cover the patch
    uint32_t pkeep = 0;
    auto prefetch = [&](int tm) {
        uint32_t b0, y0;                         // first image and first output row of the tile (uniform)
        if (g.nimg == 1) {
            b0 = fd_div((uint32_t)tm, g.d_tpi);
            y0 = ((uint32_t)tm - b0 * g.d_tpi.div) * g.rows_img;
        } else {
            b0 = (uint32_t)tm * g.nimg;
            y0 = 0;
        }
        pkeep = 0;
        if constexpr (kKeepDecode) {
            const uint32_t tile_base = (b0 * g.H + y0) * g.W * g.cdw;
            const uint32_t images_left = b0 < (uint32_t)g.B ? (uint32_t)g.B - b0 : 0u;
#pragma unroll
            for (int i = 0; i < PCH; ++i) {
                const bool inside = p_il[i] < images_left && y0 - p_ymin[i] < (uint32_t)g.H;
                const uint32_t off = inside ? tile_base + p_rel[i] : 0u;
                pp[i] = *reinterpret_cast<const uint4 *>(g.in + off);
                pkeep |= inside ? 1u << i : 0u;
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < PCH; ++i) {
            const uint32_t q = tid + i * kPNT;
            const uint32_t qq = min(q, (uint32_t)g.patch_chunks - 1);
            const uint32_t pix = qq / CPP, part = qq % CPP;
            const uint32_t t = fd_div(pix, g.d_pcol), px = pix - t * g.pcol;
            const uint32_t il = fd_div(t, g.d_prow), py = t - il * g.prow;
            const int y = (int)(y0 + py) - g.pad, x = (int)px - g.pad;
            const uint32_t b = b0 + il;
            const bool inside = q < (uint32_t)g.patch_chunks && b < (uint32_t)g.B &&
                                (unsigned)y < (unsigned)g.H && (unsigned)x < (unsigned)g.W;
            // pixels outside the image read the first chunk of the input and are masked at the commit
            const uint32_t off = inside ? ((b * g.H + y) * g.W + x) * g.cdw + part * 4 : 0u;
            pp[i] = *reinterpret_cast<const uint4 *>(g.in + off);
            pkeep |= inside ? 1u << i : 0u;
        }
    };
    auto commit = [&](uint4 *P) {
#pragma unroll
        for (int i = 0; i < PCH; ++i) {
            const uint32_t q = tid + i * kPNT;
            if (q < (uint32_t)g.patch_chunks) {
                uint32_t dst;
                if constexpr (kKeepDecode) {
                    dst = p_dst[i];
                } else {
                    const uint32_t pix = q / CPP, part = q % CPP;
                    const uint32_t t = fd_div(pix, g.d_pcol), px = pix - t * g.pcol;   // t = image * prow + patch row
                    dst = t * g.pitch + px * CPP + part;
                }
                P[dst] = keep4(pp[i], (pkeep >> i) & 1u);
            }
        }
    };
    prefetch(min(first * NH + half, tiles_m - 1));

    // ---- the block's filters: all K of 64 rows per pass, fetched once (behind the first patch's
    // loads, so that the two trips to memory overlap: a block with one or two tiles notices).  Four
    // threads share a row and take every fourth k-group of it; column nl is register column 4 (nl / 64) + nl % 4 of lane
    // (nl % 64) / 4 ---------------------------------------------------------------------------
    for (int nl0 = 64 * half; nl0 < kPBN; nl0 += 64 * NH) {
        // chunks a thread has in flight: all of a 3 x 3 filter's at once (9 * CPP k-groups over 4 threads)
        constexpr int kPatchBBatch = (9 * CPP + 3) / 4;
        const int nl = nl0 + (tid >> 2), kq = tid & 3;
        const uint32_t *brow = filt + (int64_t)min(n0 + nl, N - 1) * (g.KG * 4);
        uint4 *bdst = Bs + ((nl0 / 64) * 4 + nl % 4) * kPTX + (nl % 64) / 4;
        for (int kg = kq; kg < g.KG; kg += 4 * kPatchBBatch) {
            uint4 bv[kPatchBBatch];
#pragma unroll
            for (int u = 0; u < kPatchBBatch; ++u)
                bv[u] = *reinterpret_cast<const uint4 *>(brow + min(kg + 4 * u, g.KG - 1) * 4);
#pragma unroll
            for (int u = 0; u < kPatchBBatch; ++u)
                if (kg + 4 * u < g.KG)
                    bdst[(kg + 4 * u) * kPatchBPitch] = bv[u];
        }
    }

    // thresholds and flip word of the block's 64 columns: the same for every tile, parked in LDS
    // (the main loop needs the registers)
    if constexpr (BITS) {
        if (tid < kPBN)
            lim_s[tid] = bits.mismatch_limit(n0 + tid, N, K_true);
        if (tid < kPWords) {
            const int w = tn * kPWords + tid;
            flip_s[tid] = w < bits.Nw ? bits.flip[w] & valid_cols_mask(w, N) : 0ull;
        }
    }
    commit(P0);
    __syncthreads();

    // the lane's eight pixels: tile rows 8 ty .. 8 ty + 7 = one image row, x0 .. x0 + 7
    const int r0 = 8 * ty;
    const int il = r0 >> g.log2pix;
    const int rem = r0 & ((1 << g.log2pix) - 1);
    const int abase = (il * g.prow + (rem >> g.log2w)) * g.pitch + (rem & ((1 << g.log2w) - 1)) * CPP;
    const int wrap = g.pitch - g.kwc;            // extra chunks to the next patch row when dy advances

    int t = 0;
    for (int walk = first; walk < walks; walk += G, ++t) {
        // the half's row tile; an odd tile count leaves the last pair's second half a tile beyond
        // the matrix: it counts the last tile's patch again and stores nothing (m0 >= M)
        const int tm = walk * NH + half;
        const uint4 *P = (t & 1) ? P1 : P0;
        uint4 *Pn = (t & 1) ? P0 : P1;
        // The next patch is fetched and committed on every trip, also on the last one (where it is
        // the last tile again and never read): with both under a condition the compiler cannot
        // see that a fetch is always followed by its commit, and makes the next trip's fetch wait
        // for everything outstanding -- this trip's stores included.
        prefetch(min((walk + G) * NH + half, tiles_m - 1));

        int acc[kPTM][kPTN];

        // One k-group: operands that arrived during the previous k-group are counted while those
        // of the next one travel from LDS (two register sets alternate), as in the tile kernel.
        // The first k-group of a tile sets the counters instead of adding to them.
        auto kgroup = [&](auto first, const uint4 *pa, const uint4 *pa_next, const uint4 *pb_next, const uint4 &a0,
                          const uint4 (&b)[kPTN], uint4 &a0_next, uint4 (&b_next)[kPTN]) {
            constexpr bool kFirst = decltype(first)::value;
            uint4 a[kPTM];
            a[0] = a0;
#pragma unroll
            for (int i = 1; i < kPTM; ++i)
                a[i] = pa[i * CPP];
            a0_next = pa_next[0];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < kPTN; ++j) {
                if constexpr (kFirst)
                    xor_popc_set4(acc[0][j], a[0], b[j]);
                else
                    xor_popc_acc4(acc[0][j], a[0], b[j]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < kPTN; ++j)
                b_next[j] = pb_next[j * kPTX];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 1; i < kPTM; ++i)
#pragma unroll
                for (int j = 0; j < kPTN; ++j) {
                    if constexpr (kFirst)
                        xor_popc_set4(acc[i][j], a[i], b[j]);
                    else
                        xor_popc_acc4(acc[i][j], a[i], b[j]);
                }
        };
        // chunks from k-group k to k + 1 in the patch: 1, plus the row wrap after the last tap of a filter row
        int u = 0;
        auto advance = [&]() {
            const int step = (u + 1 == g.kwc) ? 1 + wrap : 1;
            u = (u + 1 == g.kwc) ? 0 : u + 1;
            return step;
        };
        const uint4 *pa = P + abase;
        const uint4 *pb = Bs + tx;
        uint4 a0_even, b_even[kPTN], a0_odd, b_odd[kPTN];
        a0_even = pa[0];
#pragma unroll
        for (int j = 0; j < kPTN; ++j)
            b_even[j] = pb[j * kPTX];
        // k-group 0 (and 1, if there is one) ahead of the loop, then pairs
        int k = 0;
        if (g.KG >= 2) {
            const uint4 *pa1 = pa + advance();
            const uint4 *pb1 = pb + kPatchBPitch;
            kgroup(std::true_type{}, pa, pa1, pb1, a0_even, b_even, a0_odd, b_odd);
            const bool last = 2 >= g.KG;         // no k-group behind the pair: re-read the same chunks
            const int s2 = advance();
            const uint4 *pa2 = pa1 + (last ? 0 : s2);
            const uint4 *pb2 = pb1 + (last ? 0 : kPatchBPitch);
            kgroup(std::false_type{}, pa1, pa2, pb2, a0_odd, b_odd, a0_even, b_even);
            pa = pa2;
            pb = pb2;
            k = 2;
        } else {
            kgroup(std::true_type{}, pa, pa, pb, a0_even, b_even, a0_odd, b_odd);
            k = 1;
        }
        for (; k + 1 < g.KG; k += 2) {
            const uint4 *pa1 = pa + advance();
            const uint4 *pb1 = pb + kPatchBPitch;
            kgroup(std::false_type{}, pa, pa1, pb1, a0_even, b_even, a0_odd, b_odd);
            const bool last = k + 2 >= g.KG;
            const int s2 = advance();
            const uint4 *pa2 = pa1 + (last ? 0 : s2);
            const uint4 *pb2 = pb1 + (last ? 0 : kPatchBPitch);
            kgroup(std::false_type{}, pa1, pa2, pb2, a0_odd, b_odd, a0_even, b_even);
            pa = pa2;
            pb = pb2;
        }
        if (k < g.KG)
            kgroup(std::false_type{}, pa, pa, pb, a0_even, b_even, a0_odd, b_odd);

        // The next patch goes to LDS before this tile's results are stored: loads and stores
        // complete in order, so waiting for the patch behind the stores would wait for them too.
        commit(Pn);

        // ---- epilogue -----------------------------------------------------------------
        const int m0 = tm * kPBM;
        if constexpr (BITS) {
            int lim[kPTN];
#pragma unroll
            for (int jg = 0; jg < kPWords; ++jg) {
                const int4 l4 = *reinterpret_cast<const int4 *>(&lim_s[jg * 64 + tx * 4]);
                lim[jg * 4] = l4.x, lim[jg * 4 + 1] = l4.y, lim[jg * 4 + 2] = l4.z, lim[jg * 4 + 3] = l4.w;
            }
            LaneWord lw;
            if constexpr (TN == 4)
                lw = bits.template tile_8x4<kPTY>(acc, lim, tx, ty);
            else
                lw = bits.template tile<kPTY>(acc, lim, tx, ty);
            lw.rl = r0 + (tx & 7);               // lane tx holds word tx / 8 of the lane row's pixel tx % 8
            const uint64_t word = lw.have ? ((((uint64_t)lw.hi << 32) | lw.lo) ^ flip_s[lw.wl]) : 0ull;
            const int w = tn * kPWords + lw.wl;
            if (bits.pool_log2w == 0) {
                if (lw.have && m0 + lw.rl < g.M && w < bits.Nw)
                    bits.out[(int64_t)(m0 + lw.rl) * bits.Nw + w] = word;
            } else {
                // 2x2 max-pool of +-1 values = OR of the sign bits of the tile's row pairs
                if (lw.have)
                    wt[lw.rl * kPWords + lw.wl] = word;
                __syncthreads();
                pool_tile_store<kPBM, kPWords, kPNT>(wt, bits.out, m0, n0, g.M, bits.Nw, bits.pool_log2w, tid);
            }
        } else {
#pragma unroll
            for (int i = 0; i < kPTM; ++i) {
                const int r = m0 + r0 + i;
                if (r < g.M)
                    dots.template row<kPTN, kPTX>(r, N, K_true, n0, tx, acc[i]);
            }
        }
        __syncthreads();
    }
}

// Geometry of the patch path for a shape, or false if the shape does not qualify.
static bool make_patch_geom(const uint64_t *in, int B, int H, int W, int C, int kh, int kw, int stride, int pad,
                            int H2, int W2, int tn, int nh, PatchGeom *g, size_t *lds_bytes)
{
    const int pbn = kPTX * tn;                   // filters per block tile
    if (stride != 1 || C % 128 != 0)
        return false;
    const int cpp = C / 128;
    if (cpp != 1 && cpp != 2 && cpp != 4)
        return false;
    if (W2 < 8 || W2 > 128 || (W2 & (W2 - 1)) != 0 || H2 < 1)
        return false;
    const int64_t pix_img = (int64_t)H2 * W2;
    int nimg, rows_img;
    int64_t tiles_per_img;
    if (pix_img % kPBM == 0) {
        nimg = 1;
        rows_img = kPBM / W2;
        tiles_per_img = pix_img / kPBM;
    } else if (kPBM % pix_img == 0) {
        nimg = (int)(kPBM / pix_img);
        rows_img = H2;
        tiles_per_img = 1;
    } else {
        return false;
    }
    const int64_t KG = (int64_t)kh * kw * cpp;
    if (KG > kPatchMaxKG)
        return false;
    const int prow = rows_img + kh - 1, pcol = W2 + kw - 1;
    const int64_t patch_chunks = (int64_t)nimg * prow * pcol * cpp;
    if (patch_chunks > kPatchMaxChunksPerThread * kPNT)
        return false;
    const int pitch = pcol * cpp + 1;
    const int64_t patch_lds = (int64_t)nimg * prow * pitch;
    const size_t lds = (size_t)(KG * (pbn + 1) + nh * 2 * patch_lds) * 16 + (size_t)nh * kPBM * 8 * (pbn / 64) + 16 + pbn * 4;
    // two blocks of 256 threads per CU, or one of 512 (160 KB of LDS per CU)
    if (lds > (nh == 2 ? kPatchMaxLdsWide : 64 * 1024))
        return false;
    const int cdw = 2 * (C / 64);
    if ((int64_t)B * H * W * cdw >= (1ll << 31) || (int64_t)B * pix_img >= (1ll << 31) || tiles_per_img >= (1ll << 30))
        return false;
    auto log2i = [](int64_t v) { int l = 0; while ((1ll << l) < v) ++l; return l; };
    g->in = reinterpret_cast<const uint32_t *>(in);
    g->B = B;
    g->H = H;
    g->W = W;
    g->pad = pad;
    g->M = (int)(B * pix_img);
    g->log2w = log2i(W2);
    g->log2pix = log2i(nimg == 1 ? kPBM : pix_img);
    g->nimg = nimg;
    g->rows_img = rows_img;
    g->prow = prow;
    g->pcol = pcol;
    g->pitch = pitch;
    g->patch_chunks = (int)patch_chunks;
    g->patch_lds_chunks = (int)patch_lds;
    g->kwc = kw * cpp;
    g->KG = (int)KG;
    g->cdw = cdw;
    g->d_pcol = make_fastdiv((uint32_t)pcol);
    g->d_prow = make_fastdiv((uint32_t)prow);
    g->d_tpi = make_fastdiv((uint32_t)tiles_per_img);
    *lds_bytes = lds;
    return true;
}

// Row tiles per block and blocks per filter tile for tiles_m x tiles_n tiles: the grid should be two
// blocks per compute unit (two waves per SIMD keep the vector ALUs busy), each walking the same
// number of row tiles.
static void patch_grid(int64_t tiles_m, int64_t tiles_n, int64_t slots, int64_t *G, int64_t *per_block)
{
    int64_t g = slots / tiles_n;
    g = g < 1 ? 1 : (g > tiles_m ? tiles_m : g);
    *per_block = ceil_div(tiles_m, g);
    *G = ceil_div(tiles_m, *per_block);          // the fewest blocks that still take per_block tiles each
}

// Block shape for a layer, or tn = 0 if the patch path does not apply or does not pay.
//  * 8 x 8 counters per lane (128 filters per block: half the operand reads per pair) when the layer
//    has a multiple of 128 filters, the slab fits and every block of the grid still gets a tile;
//    with 512 channels the slab of 128 filters (74 KB) only fits when the block has the CU to
//    itself: two halves of 256 threads then share it, each walking its own row tiles;
//  * else 8 x 4 (64 filters per block).
// Measured against the gathering tile kernel on the layers of the Sec. 6.3 network at batch
// 32 - 1024: 3 - 10 % faster from 512 tiles on for 128 and 256 channels (even with two row tiles
// per block); 8 x 4 counters on 512 channels (37 KB of filters to bring into LDS per block) 3 %
// slower at two row tiles per block, level at four, 2 % faster at eight.
struct PatchShape { int tn, nh; };

static PatchShape patch_shape(const uint64_t *in, const uint64_t *filt, int B, int H, int W, int C, int L2, int kh,
                              int kw, int stride, int pad, int H2, int W2, PatchGeom *g, size_t *lds)
{
    if (!aligned(in, 16) || !aligned(filt, 16))
        return PatchShape{0, 0};
    const int64_t pix_img = (int64_t)H2 * W2;
    const int cpp = C / 128;
    static const PatchShape kTry[] = {{8, 1}, {8, 2}, {4, 1}};
    for (const PatchShape &sh : kTry) {
        if (sh.nh == 2 && cpp != 4)
            continue;                            // (only instantiated for 512 channels)
        if (!make_patch_geom(in, B, H, W, C, kh, kw, stride, pad, H2, W2, sh.tn, sh.nh, g, lds))
            continue;
        const int64_t tiles_m = g->nimg == 1 ? (int64_t)B * (pix_img / kPBM) : ceil_div(B, g->nimg);
        const int64_t walks = ceil_div(tiles_m, sh.nh);
        const int64_t tiles_n = ceil_div(L2, kPTX * sh.tn);
        const int64_t slots = kPatchSlots / sh.nh;
        if (walks * tiles_n < slots || (sh.tn == 8 && L2 % 128 != 0))
            continue;
        int64_t G, per_block;
        patch_grid(walks, tiles_n, slots, &G, &per_block);
        if (cpp <= 2 || sh.nh == 2 || per_block >= 8)
            return sh;
    }
    return PatchShape{0, 0};
}

bool bconv_patch_ok(const uint64_t *in, const uint64_t *filt, int B, int H, int W, int C, int L2, int kh, int kw,
                    int stride, int pad, int H2, int W2)
{
    PatchGeom g;
    size_t lds;
    return patch_shape(in, filt, B, H, W, C, L2, kh, kw, stride, pad, H2, W2, &g, &lds).tn != 0;
}

int bconv_patch_launch(const uint64_t *in, const uint64_t *filt, int32_t *C_out, const int32_t *thr,
                       const uint64_t *flip, uint64_t *bits_out, int B, int H, int W, int C, int L2, int kh, int kw,
                       int stride, int pad, int H2, int W2, int pool_log2w, hipStream_t stream)
{
    PatchGeom g;
    size_t lds;
    const PatchShape sh = patch_shape(in, filt, B, H, W, C, L2, kh, kw, stride, pad, H2, W2, &g, &lds);
    const int tn = sh.tn;
    if (tn == 0)
        return ESP_ESHAPE;
    const int64_t pix_img = (int64_t)H2 * W2;
    const int64_t tiles_m = g.nimg == 1 ? (int64_t)B * (pix_img / kPBM) : ceil_div(B, g.nimg);
    const int64_t tiles_n = ceil_div(L2, kPTX * tn);
    if (tiles_m >= (1ll << 30) || tiles_n >= (1 << 20))
        return ESP_ESHAPE;
    int64_t G, per_block;
    patch_grid(ceil_div(tiles_m, sh.nh), tiles_n, kPatchSlots / sh.nh, &G, &per_block);
    const int K_true = kh * kw * C;
    const StoreDots dots{C_out, (L2 % 4 == 0) && aligned(C_out, 16)};
    const StoreSignBits bits{bits_out, thr, flip, (int)ceil_div(L2, 64), L2, pool_log2w};
    const dim3 grid((unsigned)(G * tiles_n)), block(kPNT * sh.nh);
    const uint32_t *f = reinterpret_cast<const uint32_t *>(filt);
    if (sh.nh == 2) {
        // 512 channels, 128 filters per block: one block of two halves per CU, more than the
        // default 64 KB of dynamic LDS (the runtime wants that announced per kernel)
        const int pch = g.patch_chunks <= 4 * kPNT ? 4 : 0;
        if (pch != 4 || C != 512)
            return ESP_ESHAPE;
#define ESP_PATCH_WIDE(BITS)                                                                                    \
        do {                                                                                                     \
            auto kern = bconv_patch_kernel<4, 4, BITS, 8, 2>;                                                    \
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                    (int)lds) != hipSuccess)                                                     \
                return ESP_ELAUNCH;                                                                              \
            hipLaunchKernelGGL(kern, grid, block, lds, stream, g, f, dots, bits, L2, K_true, (int)tiles_m,       \
                               (int)tiles_n, (int)G);                                                            \
        } while (0)
        if (bits_out)
            ESP_PATCH_WIDE(true);
        else
            ESP_PATCH_WIDE(false);
#undef ESP_PATCH_WIDE
        return launch_status();
    }
#define ESP_PATCH_LAUNCH(CPP, PCH, BITS)                                                                      \
    do {                                                                                                       \
        if (tn == 8)                                                                                           \
            hipLaunchKernelGGL((bconv_patch_kernel<CPP, PCH, BITS, 8, 1>), grid, block, lds, stream, g, f, dots,  \
                               bits, L2, K_true, (int)tiles_m, (int)tiles_n, (int)G);                          \
        else                                                                                                   \
            hipLaunchKernelGGL((bconv_patch_kernel<CPP, PCH, BITS, 4, 1>), grid, block, lds, stream, g, f, dots,  \
                               bits, L2, K_true, (int)tiles_m, (int)tiles_n, (int)G);                          \
    } while (0)
    // patch chunks per thread: as many as the channel chunks of a pixel when that covers the patch
    // (the Sec. 6.3 layers), else the maximum
    const int cpp = C / 128;
    const bool small_patch = g.patch_chunks <= cpp * kPNT;
#define ESP_PATCH_CASE(CPP)                                     \
    if (bits_out) {                                             \
        if (small_patch)                                        \
            ESP_PATCH_LAUNCH(CPP, CPP, true);                   \
        else                                                    \
            ESP_PATCH_LAUNCH(CPP, 4, true);                     \
    } else {                                                    \
        if (small_patch)                                        \
            ESP_PATCH_LAUNCH(CPP, CPP, false);                  \
        else                                                    \
            ESP_PATCH_LAUNCH(CPP, 4, false);                    \
    }
    if (cpp == 1) {
        ESP_PATCH_CASE(1)
    } else if (cpp == 2) {
        ESP_PATCH_CASE(2)
    } else {
        ESP_PATCH_CASE(4)
    }
#undef ESP_PATCH_CASE
#undef ESP_PATCH_LAUNCH
    return launch_status();
}

} // namespace esp
