// Packed unrolling (im2col), binary convolution and OR max-pooling on channel-packed
// NHWC tensors (arXiv 1705.07175, Sec. 5.2 "Convolutional layers", Fig. 3, and
// "Zero-padding for convolutions").
//
// Because tensors are packed along channels (Sec. 5.1), every tap of a sliding volume is
// a contiguous run of Cw words of the input pixel, so unrolling is a gather of whole
// words: no bit moves.  Taps outside the image become zero words (= -1).
#include <mutex>

#include "esp_internal.h"

namespace esp {

// A piece is one or two packed words moved as a unit (8- or 16-byte accesses).
typedef unsigned long long u64x2 __attribute__((ext_vector_type(2)));
template <int VEC> struct Piece;
template <> struct Piece<1> { using type = unsigned long long; };
template <> struct Piece<2> { using type = u64x2; };

// One thread per VEC-word piece of the lowered matrix.  The flat piece index is split
// into (row, tap, word) and row into (b, m, n) with multiply-shift divisions.
template <int VEC, bool STREAM_OUT>
__global__ __launch_bounds__(256)
void unroll_kernel(const uint64_t *__restrict__ in, uint64_t *__restrict__ out,
                   uint32_t total_pieces, int H, int W, int cwv /* Cw / VEC */, int kw,
                   int stride, int pad, FastDiv d_rowlen, FastDiv d_cwv, FastDiv d_kw,
                   FastDiv d_w2, FastDiv d_h2)
{
    using piece_t = typename Piece<VEC>::type;
    const piece_t *src = reinterpret_cast<const piece_t *>(in);
    piece_t *dst = reinterpret_cast<piece_t *>(out);

    // Consecutive block ids run on different XCDs, each with its own L2.  Every input pixel is
    // read kh * kw times, by the pieces of neighbouring lowered rows: dealt out by block id those
    // reads would come from all eight L2s and the input would be fetched from memory by each of
    // them.  So the grid (a multiple of 8 blocks) is cut into eight contiguous ranges of pieces,
    // one per XCD: an XCD then sweeps one eighth of the output pixels and fetches the input
    // under them once.
    const uint32_t block = xcd_contiguous_block();
    const uint32_t stride_all = gridDim.x * blockDim.x;
    for (uint32_t o = block * blockDim.x + threadIdx.x; o < total_pieces; o += stride_all) {
        const uint32_t row = fd_div(o, d_rowlen);
        const uint32_t j = o - row * d_rowlen.div;       // piece within the lowered row
        const uint32_t tap = fd_div(j, d_cwv);
        const uint32_t w = j - tap * d_cwv.div;
        const uint32_t dy = fd_div(tap, d_kw);
        const uint32_t dx = tap - dy * d_kw.div;
        const uint32_t bm = fd_div(row, d_w2);
        const uint32_t n = row - bm * d_w2.div;
        const uint32_t b = fd_div(bm, d_h2);
        const uint32_t m = bm - b * d_h2.div;
        const int y = (int)(m * stride + dy) - pad;
        const int x = (int)(n * stride + dx) - pad;
        piece_t v = piece_t(0);
        if (y >= 0 && y < H && x >= 0 && x < W)
            v = src[(((int64_t)b * H + y) * W + x) * cwv + w];
        // A large lowered matrix is written once and is kh*kw times the input: a non-temporal
        // store keeps it from displacing the input pixels (each re-read kh*kw times) from the
        // L2 (measured: 3.7 -> 6.0 TB/s).  A small one is left cacheable for the bgemm behind it.
        if (STREAM_OUT)
            __builtin_nontemporal_store(v, dst + o);
        else
            dst[o] = v;
    }
}

template <int VEC>
__global__ __launch_bounds__(256)
void bmaxpool_kernel(const uint64_t *__restrict__ in, uint64_t *__restrict__ out,
                     uint32_t total_pieces, int H, int W, int cwv, int win, int stride,
                     FastDiv d_cwv, FastDiv d_w2, FastDiv d_h2)
{
    using piece_t = typename Piece<VEC>::type;
    const piece_t *src = reinterpret_cast<const piece_t *>(in);
    piece_t *dst = reinterpret_cast<piece_t *>(out);

    const uint32_t stride_all = gridDim.x * blockDim.x;
    // (one front of blocks sweeping memory in block-id order: eight per-XCD fronts measured 5 % slower
    // on this kernel, which reads every input word once)
    for (uint32_t o = blockIdx.x * blockDim.x + threadIdx.x; o < total_pieces; o += stride_all) {
        const uint32_t pix = fd_div(o, d_cwv);
        const uint32_t w = o - pix * d_cwv.div;
        const uint32_t bm = fd_div(pix, d_w2);
        const uint32_t n = pix - bm * d_w2.div;
        const uint32_t b = fd_div(bm, d_h2);
        const uint32_t m = bm - b * d_h2.div;
        piece_t acc = piece_t(0);
        for (int dy = 0; dy < win; ++dy)
            for (int dx = 0; dx < win; ++dx) {
                const int64_t y = (int64_t)m * stride + dy;
                const int64_t x = (int64_t)n * stride + dx;
                acc |= src[(((int64_t)b * H + y) * W + x) * cwv + w]; // max of +-1 == OR of sign bits
            }
        __builtin_nontemporal_store(acc, dst + o);
    }
}

// Outputs larger than this are written with streaming (non-temporal) stores: beyond the
// combined L2 of the 8 XCDs a consumer would not find them cached anyway.
constexpr int64_t kStreamBytes = 32ll << 20;

static bool conv_shape_ok(int B, int H, int W, int C, int kh, int kw, int stride, int pad,
                          int64_t *H2, int64_t *W2)
{
    if (stride < 1 || pad < 0)
        return false;
    if ((int64_t)H + 2 * (int64_t)pad < kh || (int64_t)W + 2 * (int64_t)pad < kw)
        return false;
    *H2 = ((int64_t)H + 2 * pad - kh) / stride + 1;
    *W2 = ((int64_t)W + 2 * pad - kw) / stride + 1;
    (void)B;
    (void)C;
    return true;
}

static int unroll_launch(const uint64_t *in, uint64_t *out, int B, int H, int W, int C,
                         int kh, int kw, int stride, int pad, hipStream_t stream)
{
    int64_t H2, W2;
    if (!conv_shape_ok(B, H, W, C, kh, kw, stride, pad, &H2, &W2))
        return ESP_ESHAPE;
    const int64_t Cw = ceil_div(C, 64);
    const int64_t rows = (int64_t)B * H2 * W2;
    const int64_t total_words = rows * kh * kw * Cw;
    if (total_words >= (1ll << 31) || rows >= (1ll << 31))
        return ESP_ESHAPE;
    const bool vec2 = (Cw % 2 == 0) && aligned(in, 16) && aligned(out, 16);
    const int vec = vec2 ? 2 : 1;
    const uint32_t cwv = (uint32_t)(Cw / vec);
    const uint32_t pieces = (uint32_t)(total_words / vec);
    const FastDiv d_rowlen = make_fastdiv((uint32_t)(kh * kw) * cwv);
    const FastDiv d_cwv = make_fastdiv(cwv);
    const FastDiv d_kw = make_fastdiv((uint32_t)kw);
    const FastDiv d_w2 = make_fastdiv((uint32_t)W2);
    const FastDiv d_h2 = make_fastdiv((uint32_t)H2);
    unsigned grid = grid_for(pieces, 256);
    if (grid >= 64)
        grid = (grid + 7) / 8 * 8;       // eight equal block ranges, one per XCD (see the kernel)
    const bool stream_out = total_words * 8 > kStreamBytes;
#define ESP_UNROLL_LAUNCH(V, S)                                                                    \
    hipLaunchKernelGGL((unroll_kernel<V, S>), dim3(grid), dim3(256), 0, stream, in, out, pieces, H, \
                       W, (int)cwv, kw, stride, pad, d_rowlen, d_cwv, d_kw, d_w2, d_h2)
    if (vec2 && stream_out)
        ESP_UNROLL_LAUNCH(2, true);
    else if (vec2)
        ESP_UNROLL_LAUNCH(2, false);
    else if (stream_out)
        ESP_UNROLL_LAUNCH(1, true);
    else
        ESP_UNROLL_LAUNCH(1, false);
#undef ESP_UNROLL_LAUNCH
    return launch_status();
}

} // namespace esp

extern "C" int esp_unroll(const uint64_t *in, uint64_t *out, int B, int H, int W, int C,
                          int kh, int kw, int stride, int pad, esp_stream stream)
{
    using namespace esp;
    if (B < 0 || H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0)
        return ESP_EINVAL;
    int64_t H2, W2;
    if (!conv_shape_ok(B, H, W, C, kh, kw, stride, pad, &H2, &W2))
        return ESP_ESHAPE;
    if (B == 0)
        return ESP_OK;
    if (!in || !out)
        return ESP_EINVAL;
    if (!aligned(in, 8) || !aligned(out, 8))
        return ESP_EALIGN;
    return unroll_launch(in, out, B, H, W, C, kh, kw, stride, pad, as_stream(stream));
}

extern "C" size_t esp_bconv_workspace_bytes(int B, int H, int W, int C, int kh, int kw, int stride, int pad)
{
    using namespace esp;
    if (B <= 0 || H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0)
        return 0;
    int64_t H2, W2;
    if (!conv_shape_ok(B, H, W, C, kh, kw, stride, pad, &H2, &W2))
        return 0;
    return (size_t)((int64_t)B * H2 * W2 * kh * kw * ceil_div(C, 64) * 8);
}

extern "C" int esp_bconv_needs_workspace(int C) { return C % 128 != 0; }

namespace esp {

// log2 of W2 if a 2x2 / stride-2 max-pool can be fused behind this convolution, else 0:
// the implicit (C % 128 == 0) path only, whole pairs of image rows in every block tile.
static int pool2_log2w(int C, int64_t H2, int64_t W2)
{
    if (C % 128 != 0 || H2 < 2 || H2 % 2 != 0 || W2 < 2 || W2 > 64 || (W2 & (W2 - 1)) != 0)
        return 0;
    int l = 0;
    while ((1ll << l) < W2)
        ++l;
    return l;
}

// Shared by esp_bconv and esp_bconv_bn_sign_pack: exactly one of out_i32 / out_bits is set.
static int bconv_any(const uint64_t *in, const uint64_t *filt, int32_t *out_i32, const int32_t *thr,
                     const uint64_t *flip, uint64_t *out_bits, int B, int H, int W, int C, int L2,
                     int kh, int kw, int stride, int pad, void *workspace, size_t workspace_bytes,
                     int engine, hipStream_t stream, bool pool2 = false)
{
    if (B < 0 || H <= 0 || W <= 0 || C <= 0 || L2 <= 0 || kh <= 0 || kw <= 0 || !engine_valid(engine))
        return ESP_EINVAL;
    int64_t H2, W2;
    if (!conv_shape_ok(B, H, W, C, kh, kw, stride, pad, &H2, &W2))
        return ESP_ESHAPE;
    const int64_t K_true = (int64_t)kh * kw * C;
    if (K_true >= kMaxK)
        return ESP_ESHAPE;
    if (B == 0)
        return ESP_OK;
    if (!in || !filt || (!out_i32 && !out_bits) || (out_bits && (!thr || !flip)))
        return ESP_EINVAL;
    if (!aligned(in, 8) || !aligned(filt, 8) || !aligned(out_i32, 4) || !aligned(out_bits, 8) ||
        !aligned(thr, 4) || !aligned(flip, 8))
        return ESP_EALIGN;
    int pool_log2w = 0;
    if (pool2) {
        pool_log2w = pool2_log2w(C, H2, W2);
        if (pool_log2w == 0)
            return ESP_ESHAPE;
        if (!bconv_implicit_ok(in, filt, C))
            return ESP_EALIGN;
    }
    if (bconv_implicit_ok(in, filt, C))
        return bconv_implicit_launch(in, filt, out_i32, thr, flip, out_bits, B, H, W, C, L2, kh, kw,
                                     stride, pad, (int)H2, (int)W2, pool_log2w, engine, stream);
    // general channel counts: materialise the lowered matrix, then the plain product
    const size_t need = esp_bconv_workspace_bytes(B, H, W, C, kh, kw, stride, pad);
    if (!workspace || workspace_bytes < need)
        return ESP_EWORKSPACE;
    if (!aligned(workspace, 16))
        return ESP_EALIGN;
    uint64_t *lowered = reinterpret_cast<uint64_t *>(workspace);
    const int st = unroll_launch(in, lowered, B, H, W, C, kh, kw, stride, pad, stream);
    if (st != ESP_OK)
        return st;
    const int64_t row_words = (int64_t)kh * kw * ceil_div(C, 64);
    const int64_t M = (int64_t)B * H2 * W2;
    if (out_bits)
        return bgemm_bits_launch(lowered, filt, thr, flip, out_bits, M, L2, K_true, row_words, engine,
                                 stream);
    if (resolve_engine(engine, M, L2, K_true) == ESP_ENGINE_MFMA)
        return bgemm_mfma_launch(lowered, filt, out_i32, nullptr, nullptr, nullptr, M, L2, K_true, row_words,
                                 stream);
    return bgemm_launch(lowered, filt, out_i32, M, L2, K_true, row_words, stream);
}

} // namespace esp

extern "C" int esp_bconv(const uint64_t *in, const uint64_t *filt, int32_t *out,
                         int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                         void *workspace, size_t workspace_bytes, esp_stream stream)
{
    if (B > 0 && !out)
        return ESP_EINVAL;
    return esp::bconv_any(in, filt, out, nullptr, nullptr, nullptr, B, H, W, C, L2, kh, kw, stride, pad,
                          workspace, workspace_bytes, ESP_ENGINE_XOR_POPCOUNT, esp::as_stream(stream));
}

// ---- esp_bconv for callers that cannot allocate -------------------------------------
// The lowered matrix of esp_bconv's general path lives in `scratch`, a fixed array in the
// code object: each GPU that loads the library holds its own copy until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress; the address it
// returns for the current device is what the kernels get.
constexpr size_t kScratchBytes = ESP_BCONV_NOALLOC_MAX_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace esp {

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static void *g_scratch_ptr[kMaxDevices];      // per device: where that GPU's copy of `scratch` lies

// Address of the current device's `scratch`, looked up once per device.
static int scratch_of_current_device(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return ESP_ELAUNCH;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p)
            return ESP_ELAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return ESP_OK;
}

} // namespace esp

extern "C" int esp_bconv_noalloc(const uint64_t *in, const uint64_t *filt, int32_t *out,
                                 int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                                 esp_stream stream)
{
    using namespace esp;
    if (B > 0 && !out)
        return ESP_EINVAL;
    // shapes are judged before the scratch is looked up, so that argument errors come back the
    // same way as from esp_bconv
    const size_t need = esp_bconv_workspace_bytes(B, H, W, C, kh, kw, stride, pad);
    const bool lowered = B > 0 && need > 0 && in && filt && !bconv_implicit_ok(in, filt, C);
    if (lowered && need > kScratchBytes)
        return ESP_EWORKSPACE;
    void *ws = nullptr;
    if (lowered) {
        const int st = scratch_of_current_device(&ws);
        if (st != ESP_OK)
            return st;
    }
    return bconv_any(in, filt, out, nullptr, nullptr, nullptr, B, H, W, C, L2, kh, kw, stride, pad, ws,
                     ws ? kScratchBytes : 0, ESP_ENGINE_XOR_POPCOUNT, as_stream(stream));
}

extern "C" int esp_bconv_mfma(const uint64_t *in, const uint64_t *filt, int32_t *out,
                              int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                              void *workspace, size_t workspace_bytes, esp_stream stream)
{
    if (B > 0 && !out)
        return ESP_EINVAL;
    return esp::bconv_any(in, filt, out, nullptr, nullptr, nullptr, B, H, W, C, L2, kh, kw, stride, pad,
                          workspace, workspace_bytes, ESP_ENGINE_MFMA, esp::as_stream(stream));
}

extern "C" int esp_bconv_bn_sign_pack(const uint64_t *in, const uint64_t *filt, const int32_t *thr,
                                      const uint64_t *flip, uint64_t *out,
                                      int B, int H, int W, int C, int L2, int kh, int kw, int stride,
                                      int pad, void *workspace, size_t workspace_bytes, int engine,
                                      esp_stream stream)
{
    if (B > 0 && (!out || !thr || !flip))
        return ESP_EINVAL;
    return esp::bconv_any(in, filt, nullptr, thr, flip, out, B, H, W, C, L2, kh, kw, stride, pad,
                          workspace, workspace_bytes, engine, esp::as_stream(stream));
}

extern "C" int esp_bconv_pool2_fusable(int H, int W, int C, int kh, int kw, int stride, int pad)
{
    using namespace esp;
    if (H <= 0 || W <= 0 || C <= 0 || kh <= 0 || kw <= 0)
        return 0;
    int64_t H2, W2;
    if (!conv_shape_ok(1, H, W, C, kh, kw, stride, pad, &H2, &W2))
        return 0;
    return pool2_log2w(C, H2, W2) != 0;
}

extern "C" int esp_bconv_bn_sign_pack_pool2(const uint64_t *in, const uint64_t *filt, const int32_t *thr,
                                            const uint64_t *flip, uint64_t *out,
                                            int B, int H, int W, int C, int L2, int kh, int kw, int stride,
                                            int pad, int engine, esp_stream stream)
{
    if (B > 0 && (!out || !thr || !flip))
        return ESP_EINVAL;
    return esp::bconv_any(in, filt, nullptr, thr, flip, out, B, H, W, C, L2, kh, kw, stride, pad, nullptr, 0,
                          engine, esp::as_stream(stream), true);
}

namespace esp {

// Correction matrix of Sec. 5.2 "Zero-padding for convolutions": the convolution of the
// layer's weights with a tensor that is 0 inside the image and +1 in the padding ring.
// corr[m][n][l2] = sum over the taps of output pixel (m, n) that fall outside the image of
// sum_c F[l2][dy][dx][c] = 2 * popcount(filter words of that tap) - C.
__global__ __launch_bounds__(256)
void pad_correction_kernel(const uint64_t *__restrict__ filt, int32_t *__restrict__ corr, int H, int W,
                           int C, int Cw, int L2, int kh, int kw, int stride, int pad, int H2, int W2)
{
    const int64_t total = (int64_t)H2 * W2 * L2;
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= total)
        return;
    const int l2 = (int)(o % L2);
    const int n = (int)((o / L2) % W2);
    const int m = (int)(o / ((int64_t)L2 * W2));
    int acc = 0;
    for (int dy = 0; dy < kh; ++dy)
        for (int dx = 0; dx < kw; ++dx) {
            const int y = m * stride + dy - pad, x = n * stride + dx - pad;
            if (y >= 0 && y < H && x >= 0 && x < W)
                continue;
            const uint64_t *f = filt + (((int64_t)l2 * kh + dy) * kw + dx) * Cw;
            int ones = 0;
            for (int w = 0; w < Cw; ++w)
                ones += __popcll(f[w]);
            acc += 2 * ones - C;
        }
    corr[o] = acc;
}

// Output pixels whose sliding volume leaves the image: rows [0, mt) and [mb, H2) entirely,
// and columns [0, nl) and [nr, W2) of the rows in between.
struct BorderMap {
    int W2, mt, mb, nl, nr, side, top, mid, count;
};

static BorderMap make_border(int H, int W, int kh, int kw, int stride, int pad, int H2, int W2)
{
    auto first_rows = [&](int n2) { int t = (pad + stride - 1) / stride; return t < n2 ? t : n2; };
    auto last_start = [&](int size, int k, int n2, int lo) {
        // first index whose window ends beyond the image
        int64_t t = ((int64_t)size - k + pad) / stride + 1;
        if ((int64_t)size - k + pad < 0)
            t = 0;
        if (t < lo)
            t = lo;
        return (int)(t < n2 ? t : n2);
    };
    BorderMap b;
    b.W2 = W2;
    b.mt = first_rows(H2);
    b.mb = last_start(H, kh, H2, b.mt);
    b.nl = first_rows(W2);
    b.nr = last_start(W, kw, W2, b.nl);
    b.side = b.nl + (W2 - b.nr);
    b.top = b.mt * W2;
    b.mid = (b.mb - b.mt) * b.side;
    b.count = b.top + b.mid + (H2 - b.mb) * W2;
    return b;
}

// x[b][pixel][:] += corr[pixel][:] for the border pixels only (the correction is zero
// elsewhere); VEC int32 per thread.
template <int VEC>
__global__ __launch_bounds__(256)
void add_correction_kernel(int32_t *__restrict__ x, const int32_t *__restrict__ corr, int B,
                           int pixels, int L2, BorderMap bm)
{
    const int lv = L2 / VEC;
    const int64_t total = (int64_t)B * bm.count * lv;
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (o >= total)
        return;
    const int cv = (int)(o % lv);
    const int idx = (int)((o / lv) % bm.count);
    const int b = (int)(o / ((int64_t)lv * bm.count));
    int m, n;
    if (idx < bm.top) {
        m = idx / bm.W2;
        n = idx - m * bm.W2;
    } else if (idx < bm.top + bm.mid) {
        const int r = idx - bm.top;
        const int q = r / bm.side, j = r - q * bm.side;
        m = bm.mt + q;
        n = j < bm.nl ? j : bm.nr + (j - bm.nl);
    } else {
        const int r = idx - bm.top - bm.mid;
        const int q = r / bm.W2;
        m = bm.mb + q;
        n = r - q * bm.W2;
    }
    const int64_t pix = (int64_t)m * bm.W2 + n;
    int32_t *px = x + ((int64_t)b * pixels + pix) * L2 + cv * VEC;
    const int32_t *pc = corr + pix * L2 + cv * VEC;
    if (VEC == 4) {
        int4 v = *reinterpret_cast<int4 *>(px);
        const int4 c = *reinterpret_cast<const int4 *>(pc);
        v.x += c.x;
        v.y += c.y;
        v.z += c.z;
        v.w += c.w;
        *reinterpret_cast<int4 *>(px) = v;
    } else {
        *px += *pc;
    }
}

} // namespace esp

extern "C" int esp_pad_correction(const uint64_t *filt, int32_t *corr, int H, int W, int C, int L2,
                                  int kh, int kw, int stride, int pad, esp_stream stream)
{
    using namespace esp;
    if (H <= 0 || W <= 0 || C <= 0 || L2 <= 0 || kh <= 0 || kw <= 0)
        return ESP_EINVAL;
    int64_t H2, W2;
    if (!conv_shape_ok(1, H, W, C, kh, kw, stride, pad, &H2, &W2))
        return ESP_ESHAPE;
    if (!filt || !corr)
        return ESP_EINVAL;
    if (!aligned(filt, 8) || !aligned(corr, 4))
        return ESP_EALIGN;
    const int64_t total = H2 * W2 * L2;
    if (total >= (1ll << 38))
        return ESP_ESHAPE;
    hipLaunchKernelGGL(pad_correction_kernel, dim3(grid_for(total, 256)), dim3(256), 0, as_stream(stream),
                       filt, corr, H, W, C, (int)ceil_div(C, 64), L2, kh, kw, stride, pad, (int)H2, (int)W2);
    return launch_status();
}

extern "C" int esp_add_pad_correction(int32_t *x, const int32_t *corr, int B, int H, int W, int L2,
                                      int kh, int kw, int stride, int pad, esp_stream stream)
{
    using namespace esp;
    if (B < 0 || H <= 0 || W <= 0 || L2 <= 0 || kh <= 0 || kw <= 0)
        return ESP_EINVAL;
    int64_t H2, W2;
    if (!conv_shape_ok(B, H, W, 1, kh, kw, stride, pad, &H2, &W2))
        return ESP_ESHAPE;
    if (B == 0)
        return ESP_OK;
    if (!x || !corr)
        return ESP_EINVAL;
    if (!aligned(x, 4) || !aligned(corr, 4))
        return ESP_EALIGN;
    if (H2 * W2 >= (1ll << 31))
        return ESP_ESHAPE;
    const BorderMap bm = make_border(H, W, kh, kw, stride, pad, (int)H2, (int)W2);
    if (bm.count == 0)
        return ESP_OK;
    const bool vec4 = (L2 % 4 == 0) && aligned(x, 16) && aligned(corr, 16);
    const int64_t total = (int64_t)B * bm.count * (vec4 ? L2 / 4 : L2);
    if (total >= (1ll << 38))
        return ESP_ESHAPE;
    if (vec4)
        hipLaunchKernelGGL((add_correction_kernel<4>), dim3(grid_for(total, 256)), dim3(256), 0,
                           as_stream(stream), x, corr, B, (int)(H2 * W2), L2, bm);
    else
        hipLaunchKernelGGL((add_correction_kernel<1>), dim3(grid_for(total, 256)), dim3(256), 0,
                           as_stream(stream), x, corr, B, (int)(H2 * W2), L2, bm);
    return launch_status();
}

extern "C" int esp_bmaxpool(const uint64_t *in, uint64_t *out, int B, int H, int W, int C,
                            int win, int stride, esp_stream stream)
{
    using namespace esp;
    if (B < 0 || H <= 0 || W <= 0 || C <= 0 || win <= 0)
        return ESP_EINVAL;
    if (stride < 1 || win > H || win > W)
        return ESP_ESHAPE;
    if (B == 0)
        return ESP_OK;
    if (!in || !out)
        return ESP_EINVAL;
    if (!aligned(in, 8) || !aligned(out, 8))
        return ESP_EALIGN;
    const int64_t H2 = (H - win) / stride + 1;
    const int64_t W2 = (W - win) / stride + 1;
    const int64_t Cw = ceil_div(C, 64);
    const int64_t total_words = (int64_t)B * H2 * W2 * Cw;
    if (total_words >= (1ll << 31))
        return ESP_ESHAPE;
    const bool vec2 = (Cw % 2 == 0) && aligned(in, 16) && aligned(out, 16);
    const int vec = vec2 ? 2 : 1;
    const uint32_t cwv = (uint32_t)(Cw / vec);
    const uint32_t pieces = (uint32_t)(total_words / vec);
    const FastDiv d_cwv = make_fastdiv(cwv);
    const FastDiv d_w2 = make_fastdiv((uint32_t)W2);
    const FastDiv d_h2 = make_fastdiv((uint32_t)H2);
    const unsigned grid = grid_for(pieces, 256);
    if (vec2)
        hipLaunchKernelGGL((bmaxpool_kernel<2>), dim3(grid), dim3(256), 0, as_stream(stream), in, out,
                           pieces, H, W, (int)cwv, win, stride, d_cwv, d_w2, d_h2);
    else
        hipLaunchKernelGGL((bmaxpool_kernel<1>), dim3(grid), dim3(256), 0, as_stream(stream), in, out,
                           pieces, H, W, (int)cwv, win, stride, d_cwv, d_w2, d_h2);
    return launch_status();
}
