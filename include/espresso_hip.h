/*
 * espresso_hip.h -- C ABI of the MI355X (gfx950) binary-network forward library.
 *
 * The library implements the bit-packed forward path of Espresso
 * (arXiv 1705.07175): binary dense and convolutional layers whose dot products
 * are evaluated on 64-bit packed words (Sec. 4.2, Eq. 2), plus the supporting
 * steps around them (bit-packing, unrolling, batch-norm + sign re-packing,
 * pooling, and the real-valued first layer).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  * Encoding (Sec. 4.1): -1 is bit 0, +1 is bit 1.  sign(x) = +1 iff x >= 0
 *    (Eq. 1), so 0.0 and -0.0 give bit 1 and NaN gives bit 0.
 *  * Packing (Sec. 4.2, Sec. 5.1): values are packed along their last
 *    dimension (K for matrices, the channel l for NHWC tensors) into uint64
 *    words.  Element k lives in word k/64, bit k%64, least significant bit
 *    first.  A row of K values takes Kw = ceil(K/64) words; the unused high
 *    bits of its last word are 0 in every buffer the library writes and MUST
 *    be 0 in every packed buffer it reads.
 *  * Tensors (Sec. 5.1): row-major with interleaved channels, element (m,n,l)
 *    at (m*N+n)*L+l, with the batch index prepended: [B][H][W][C] ("NHWC").
 *    Dense weights and convolution filters hold one neuron/filter per row.
 *  * Memory: unless a parameter is marked HOST, every pointer is DEVICE memory
 *    owned by the caller (the paper pre-allocates all memory, Sec. 3
 *    "Technical highlights"; here the caller does).  The library never
 *    allocates, frees or synchronises.  Outputs are overwritten completely,
 *    inputs are never modified, inputs and outputs must not overlap.
 *  * Execution: every device entry point only enqueues kernels on `stream`
 *    (a hipStream_t passed as void*; NULL is the default stream) and returns.
 *  * Errors: the return value is ESP_OK or a negative esp_status.  Nothing is
 *    enqueued when an error is returned.  The library never throws, aborts or
 *    prints.  uint64 buffers must be 8-byte aligned, int32/float buffers
 *    4-byte aligned (ESP_EALIGN otherwise); 16-byte alignment of every base
 *    pointer enables the fastest paths.
 *  * Sizes: 0 < K < 2^30 so that |dot| fits int32; a dimension of 0 rows
 *    (rows, M, B) is accepted and does nothing; other non-positive
 *    dimensions give ESP_EINVAL.
 */
#ifndef ESPRESSO_HIP_H
#define ESPRESSO_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *esp_stream; /* hipStream_t; NULL = default stream */

enum esp_status {
    ESP_OK = 0,
    ESP_EINVAL = -1,     /* null pointer, negative or zero dimension              */
    ESP_EALIGN = -2,     /* a buffer is not aligned for its element type          */
    ESP_ESHAPE = -3,     /* shapes inconsistent (kernel larger than padded input, */
                         /* stride < 1, pad < 0, pooled size 0, K >= 2^30, ...)   */
    ESP_EWORKSPACE = -4, /* workspace missing or too small                        */
    ESP_ELAUNCH = -5     /* the HIP runtime refused a launch                      */
};

/* Which units evaluate the binary contraction of the fused / convolution     */
/* entry points that take an `engine` argument.  Results are identical.       */
enum esp_engine {
    ESP_ENGINE_XOR_POPCOUNT = 0, /* vector ALU: v_xor + v_bcnt (the paper's XNOR/bit-count) */
    ESP_ENGINE_MFMA = 1,         /* matrix cores: bits expanded to 4-bit float operands      */
    ESP_ENGINE_AUTO = 2          /* matrix cores when the product fills the chip with their  */
                                 /* 256 x 128 tiles, the vector ALU otherwise                */
};
/* On the vector ALU a product is tiled (128 x 128 down to 32 x 64 outputs per block) or, when */
/* it has few rows (a network evaluated on one or a few images), split over K instead; with    */
/* ESP_ENGINE_MFMA every product goes to the matrix cores whatever its size.                   */

/* Human-readable name of a status code (static string, never NULL). */
const char *esp_strerror(int status);

/* Library version, major*10000 + minor*100 + patch. */
int esp_version(void);

/* ------------------------------------------------------------------------- */
/* pack: sign (Eq. 1) + bit-packing along the row (Sec. 4.2; the row-packing  */
/* kernel of Sec. 6.2 "Optimized kernels").                                   */
/*   src  float [rows][k]           dst  uint64 [rows][ceil(k/64)]            */
/* Weights are packed once at load time, not per forward (Sec. 6.2 "Binary    */
/* optimized layers").  An NHWC tensor is packed along channels by passing    */
/* rows = B*H*W, k = C.                                                        */
/* ------------------------------------------------------------------------- */
int esp_pack_f32(const float *src, uint64_t *dst, int64_t rows, int64_t k, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* bgemm: binary matrix product (Sec. 4.2, Eq. 2; kernel design prior art in  */
/* Sec. 5.2 "Efficient Matrix multiplication", sizes of Sec. 6.1).            */
/*   A  uint64 [M][Kw]   packed activations, one input row per row            */
/*   B  uint64 [N][Kw]   packed weights, one neuron per row                   */
/*   C  int32  [M][N]    C[m][n] = K - 2 * sum_w popcount(A[m][w] XOR B[n][w])*/
/* which equals the dot product of the two +-1 rows of true length K          */
/* (Kw = ceil(K/64); zero tail bits cancel in the XOR).  Eq. 2 as printed     */
/* counts matches and subtracts them, which would negate the result; the      */
/* mismatch form above is the one that equals the +-1 dot product.            */
/* Any M >= 0, N > 0; small M (matrix-vector, Sec. 6.2 "Optimized kernels")   */
/* is dispatched to a bandwidth-oriented kernel.                              */
/* ------------------------------------------------------------------------- */
int esp_bgemm(const uint64_t *A, const uint64_t *B, int32_t *C,
              int64_t M, int64_t N, int64_t K, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* bgemm_mfma: the same product as esp_bgemm (identical int32 results),       */
/* evaluated on the matrix cores instead of XOR + popcount: the packed bits   */
/* are expanded in registers to 4-bit floating-point operands of the          */
/* block-scaled MFMA and accumulated exactly in fp32.  A measured alternative */
/* for the dense contraction; K < 2^24.                                       */
/* ------------------------------------------------------------------------- */
int esp_bgemm_mfma(const uint64_t *A, const uint64_t *B, int32_t *C,
                   int64_t M, int64_t N, int64_t K, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* unroll: packed im2col (Sec. 5.2 "Convolutional layers", Fig. 3).           */
/*   in   uint64 [B][H][W][Cw]                  Cw = ceil(C/64)               */
/*   out  uint64 [B*H2*W2][kh*kw*Cw]            H2 = (H+2*pad-kh)/stride+1    */
/* Row (b*H2+m)*W2+n holds the sliding volume in[b][m*s-p .. +kh][n*s-p ..    */
/* +kw][:] tap by tap: word (dy*kw+dx)*Cw + w.  Taps outside the image are    */
/* all-zero words, i.e. the value -1 (Sec. 5.2 "Zero-padding for              */
/* convolutions": the border is treated as -1).                               */
/* ------------------------------------------------------------------------- */
int esp_unroll(const uint64_t *in, uint64_t *out, int B, int H, int W, int C,
               int kh, int kw, int stride, int pad, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* bconv: binary convolution = unroll + bgemm (Sec. 5.2, Fig. 3); the output  */
/* rows are already NHWC so no lifting step exists.                           */
/*   in    uint64 [B][H][W][Cw]                                               */
/*   filt  uint64 [L2][kh][kw][Cw]   one filter per row, taps in unroll order */
/*   out   int32  [B][H2][W2][L2]    +-1 cross-correlation over kh*kw*C taps, */
/*                                    border = -1                             */
/*   workspace  device scratch of at least esp_bconv_workspace_bytes(...)     */
/*              bytes, 16-byte aligned (holds the lowered matrix).  When C is */
/*              a multiple of 128 (esp_bconv_needs_workspace(C) == 0) and in, */
/*              filt are 16-byte aligned, the sliding volumes are gathered    */
/*              inside the product kernel, no lowered matrix is written and   */
/*              the workspace is not touched (it may then be NULL).           */
/* ------------------------------------------------------------------------- */
size_t esp_bconv_workspace_bytes(int B, int H, int W, int C, int kh, int kw, int stride, int pad);

int esp_bconv_needs_workspace(int C);

int esp_bconv(const uint64_t *in, const uint64_t *filt, int32_t *out,
              int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
              void *workspace, size_t workspace_bytes, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* bconv_noalloc: esp_bconv for callers that cannot allocate device memory    */
/* (code under HIP graph capture, tight serving loops, harnesses that forbid  */
/* hipMalloc) and therefore cannot bring a workspace.  Same arguments without */
/* the workspace, same results.  The lowered matrix of the general path (C    */
/* not a multiple of 128, or in / filt not 16-byte aligned) is written to a   */
/* fixed scratch array inside the library, ESP_BCONV_NOALLOC_MAX_BYTES =      */
/* 16 MiB per GPU, held from library load until the process ends; a shape     */
/* whose esp_bconv_workspace_bytes(...) exceeds it returns ESP_EWORKSPACE and */
/* enqueues nothing.  The call allocates and frees nothing and does not       */
/* synchronise.  The first call on a device looks up that device's copy of    */
/* the array (a runtime query, no allocation): make it once outside a graph   */
/* capture.  All calls on one GPU share the array: two calls may overlap only */
/* if they are ordered on one stream (or otherwise serialised); calls on      */
/* different streams of the same GPU race on it.  Nothing in the array needs  */
/* clearing between calls: every word the product reads is written by the     */
/* same call first.  Errors otherwise as esp_bconv (ESP_ELAUNCH if the        */
/* device's array cannot be found).                                           */
/* ------------------------------------------------------------------------- */
#define ESP_BCONV_NOALLOC_MAX_BYTES ((size_t)16 << 20)

int esp_bconv_noalloc(const uint64_t *in, const uint64_t *filt, int32_t *out,
                      int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                      esp_stream stream);

/* ------------------------------------------------------------------------- */
/* bn_fold (HOST function, run once per layer at load time): folds inference  */
/* batch-norm followed by sign (Sec. 5.2 lists the batch-norm layer; Eq. 1)   */
/* into one integer threshold per channel.  With                              */
/*   y(x) = gamma*(x-mean)/sqrt(var+eps) + beta   evaluated in double, left   */
/*   to right, no fused multiply-add,                                         */
/* the outputs satisfy, for every integer |x| <= 2^30,                        */
/*   (y(x) >= 0)  ==  (x >= thr[c]) XOR flipbit(c)                            */
/* where flipbit(c) is bit c%64 of flip[c/64].                                */
/*   gamma, beta, mean, var   HOST float [C]                                  */
/*   thr   HOST int32 [C]       flip  HOST uint64 [ceil(C/64)]                */
/* ------------------------------------------------------------------------- */
int esp_bn_fold(const float *gamma, const float *beta, const float *mean, const float *var,
                float eps, int C, int32_t *thr, uint64_t *flip);

/* ------------------------------------------------------------------------- */
/* bn_sign_pack: batch-norm + sign + re-pack of an integer layer output (the  */
/* bit-packing sign activation of Sec. 6.3 "Bit-packing"), using the folded   */
/* threshold:  bit c of row r = (x[r][c] >= thr[c]) XOR flipbit(c).           */
/*   x  int32 [rows][C]   thr int32 [C]   flip uint64 [Cw]   out uint64 [rows][Cw] */
/* ------------------------------------------------------------------------- */
int esp_bn_sign_pack(const int32_t *x, const int32_t *thr, const uint64_t *flip,
                     uint64_t *out, int64_t rows, int C, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* Fused layer outputs: the folded threshold of esp_bn_fold applied in the    */
/* epilogue of the product, so that a binary layer writes the packed sign     */
/* bits of the next layer directly and its int32 pre-activations never reach  */
/* memory (Sec. 6.3 "Bit-packing" names this re-packing as the growing cost   */
/* of convolutional layers).  Results are identical to esp_bgemm / esp_bconv  */
/* followed by esp_bn_sign_pack.                                              */
/*   bgemm_bn_sign_pack:  A [M][Kw], B [N][Kw] -> out uint64 [M][ceil(N/64)]  */
/*   bconv_bn_sign_pack:  in [B][H][W][Cw], filt [L2][kh][kw][Cw]             */
/*                        -> out uint64 [B][H2][W2][ceil(L2/64)]              */
/*   thr int32 [N or L2], flip uint64 [ceil(N or L2 / 64)]; workspace as for  */
/*   esp_bconv; engine is an esp_engine (ESP_EINVAL otherwise; the MFMA       */
/*   engine needs K < 2^24).  esp_bconv_mfma is esp_bconv on the matrix cores.*/
/* ------------------------------------------------------------------------- */
int esp_bgemm_bn_sign_pack(const uint64_t *A, const uint64_t *B, const int32_t *thr,
                           const uint64_t *flip, uint64_t *out,
                           int64_t M, int64_t N, int64_t K, int engine, esp_stream stream);

int esp_bconv_bn_sign_pack(const uint64_t *in, const uint64_t *filt, const int32_t *thr,
                           const uint64_t *flip, uint64_t *out,
                           int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                           void *workspace, size_t workspace_bytes, int engine, esp_stream stream);

int esp_bconv_mfma(const uint64_t *in, const uint64_t *filt, int32_t *out,
                   int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                   void *workspace, size_t workspace_bytes, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* bconv_bn_sign_pack_pool2: esp_bconv_bn_sign_pack followed by the 2x2,      */
/* stride-2 esp_bmaxpool, in one kernel.  In the network of Sec. 6.3 pooling  */
/* acts on the +-1 activations, where the maximum is the OR of the sign bits; */
/* a block tile that holds whole pairs of image rows ORs them before storing, */
/* so the unpooled activations never reach memory.                            */
/*   out uint64 [B][H2/2][W2/2][ceil(L2/64)]; other arguments as above; no    */
/*   workspace.  Only for shapes where esp_bconv_pool2_fusable returns 1:     */
/*   C a multiple of 128, H2 even, W2 a power of two in [2, 64]; otherwise    */
/*   ESP_ESHAPE (ESP_EALIGN if in / filt are not 16-byte aligned) and the     */
/*   caller chains the two separate calls.  Results are identical to them.    */
/* ------------------------------------------------------------------------- */
int esp_bconv_pool2_fusable(int H, int W, int C, int kh, int kw, int stride, int pad);

int esp_bconv_bn_sign_pack_pool2(const uint64_t *in, const uint64_t *filt, const int32_t *thr,
                                 const uint64_t *flip, uint64_t *out,
                                 int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                                 int engine, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* Zero-padding correction (Sec. 5.2 "Zero-padding for convolutions"): the    */
/* binary convolution above treats the border as -1; a zero-padded ("same")   */
/* convolution is obtained by adding a correction matrix that depends only on */
/* the weights.                                                               */
/*   pad_correction (once per layer, at load time):                           */
/*     corr int32 [H2][W2][L2] = convolution of the weights with a tensor     */
/*     that is 0 inside the H x W image and +1 in the padding ring; it is     */
/*     non-zero only where a sliding volume leaves the image.                 */
/*   add_pad_correction: x[b][m][n][:] += corr[m][n][:] for every image b, IN */
/*     PLACE on the int32 result of esp_bconv ([B][H2][W2][L2]); only the     */
/*     border pixels are touched.  After it, x equals the convolution with    */
/*     zero padding.  The geometry arguments must be those of the bconv call. */
/* ------------------------------------------------------------------------- */
int esp_pad_correction(const uint64_t *filt, int32_t *corr, int H, int W, int C, int L2,
                       int kh, int kw, int stride, int pad, esp_stream stream);

int esp_add_pad_correction(int32_t *x, const int32_t *corr, int B, int H, int W, int L2,
                           int kh, int kw, int stride, int pad, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* bmaxpool: max-pooling of +-1 activations on packed words (pooling layer of */
/* Sec. 5.2): the maximum of +-1 values is the bitwise OR of their bits.      */
/*   in  uint64 [B][H][W][Cw]   out uint64 [B][H2][W2][Cw]                    */
/*   H2 = (H-win)/stride + 1 (floor), no padding.                             */
/* ------------------------------------------------------------------------- */
int esp_bmaxpool(const uint64_t *in, uint64_t *out, int B, int H, int W, int C,
                 int win, int stride, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* Real-valued first layer (the non-binary variant of a layer, Sec. 3; the    */
/* networks of Sec. 6.2 / 6.3 receive real-valued images).  fp32 arithmetic.  */
/*   dense:  X float [M][K], W float [N][K] (+-1 values), Y float [M][N]      */
/*   conv :  in float [B][H][W][C], filt float [L2][kh][kw][C] (+-1 values),  */
/*           out float [B][H2][W2][L2], zero padding                          */
/* The weights of these layers are the +-1 of a binary network held as floats */
/* (Sec. 4.3: real-valued input, binary weights).  esp_dense_f32 is plain     */
/* fp32 for any weight values; the fused dense layer (more than 4 rows) and   */
/* the 3x3x3 stride-1 convolution rely on the +-1: they run on the bf16       */
/* matrix cores with every input split exactly into three bf16 terms and the  */
/* weights taken as bf16, which is exact for +-1 (any other weight would be   */
/* cut to 8 significant bits); sums are accumulated in fp32 either way.       */
/* ------------------------------------------------------------------------- */
int esp_dense_f32(const float *X, const float *W, float *Y,
                  int64_t M, int64_t N, int64_t K, esp_stream stream);

int esp_conv_f32(const float *in, const float *filt, float *out,
                 int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                 esp_stream stream);

/* ------------------------------------------------------------------------- */
/* bn_fold_f32 (HOST function, once per layer at load time): the same fold as */
/* esp_bn_fold for float pre-activations.  With y(x) as defined there (double,*/
/* left to right), the outputs satisfy for every finite float x               */
/*   (y(x) >= 0)  ==  (sgn[c] * x >= thr[c])      sgn[c] is +1 or -1,         */
/* thr[c] = -inf / +inf encode a bit that is constant 1 / 0.                  */
/*   gamma, beta, mean, var   HOST float [C]     thr, sgn   HOST float [C]    */
/*                                                                            */
/* bn_sign_pack_f32: bit c of row r = (sgn[c] * x[r][c] >= thr[c]); NaN -> 0. */
/*   x float [rows][C]   thr, sgn DEVICE float [C]   out uint64 [rows][Cw]    */
/*                                                                            */
/* conv_f32_bn_sign_pack: esp_conv_f32 followed by esp_bn_sign_pack_f32 in    */
/* one pass; `bits` uint64 [B][H2][W2][ceil(L2/64)] is always written, `pre`  */
/* (float [B][H2][W2][L2], the pre-activations) only if not NULL.  For filter */
/* shapes without a fused kernel `pre` is required as scratch                 */
/* (ESP_EWORKSPACE if NULL).                                                  */
/*                                                                            */
/* dense_f32_bn_sign_pack: esp_dense_f32 followed by esp_bn_sign_pack_f32 in  */
/* one kernel; `bits` uint64 [M][ceil(N/64)] is always written, `pre` (float  */
/* [M][N], the pre-activations) only if not NULL.                             */
/*                                                                            */
/* dense_f32_bw_bn_sign_pack: the same layer with its +-1 weights bit-packed  */
/* (Wbits uint64 [N][ceil(K/64)] as esp_pack_f32 writes them: bit 1 = +1,     */
/* zero tail; Sec. 6.2 "Binary optimized layers": weights are packed once at  */
/* load time) -- 1/32 of the weight memory and traffic, which is most of what */
/* this layer costs when a network is evaluated one input at a time.  The     */
/* pre-activations are fp32 sums of +-x[k] (same tolerance as the float form, */
/* the summation order differs).  K < 2^30.                                   */
/* ------------------------------------------------------------------------- */
int esp_bn_fold_f32(const float *gamma, const float *beta, const float *mean, const float *var,
                    float eps, int C, float *thr, float *sgn);

int esp_bn_sign_pack_f32(const float *x, const float *thr, const float *sgn,
                         uint64_t *out, int64_t rows, int C, esp_stream stream);

int esp_dense_f32_bn_sign_pack(const float *X, const float *W, const float *thr, const float *sgn,
                               uint64_t *bits, float *pre, int64_t M, int64_t N, int64_t K,
                               esp_stream stream);

int esp_dense_f32_bw_bn_sign_pack(const float *X, const uint64_t *Wbits, const float *thr,
                                  const float *sgn, uint64_t *bits, float *pre, int64_t M, int64_t N,
                                  int64_t K, esp_stream stream);

int esp_conv_f32_bn_sign_pack(const float *in, const float *filt, const float *thr, const float *sgn,
                              uint64_t *bits, float *pre,
                              int B, int H, int W, int C, int L2, int kh, int kw, int stride, int pad,
                              esp_stream stream);

/* ------------------------------------------------------------------------- */
/* Binary first layer on 8-bit fixed-precision input by bit-planes (Sec. 4.3, */
/* Eq. 3; Sec. 6.2 "First-layer binary optimization": the input is split into */
/* 8 rows and the products are recombined by a weighted sum).  Exact integer  */
/* result  y[r][n] = sum_k x[r][k] * w[n][k],  x in 0..255, w = +-1.          */
/*   bitplane_pack_u8:  x uint8 [outer][inner][k] ->                          */
/*                      planes uint64 [outer][8][inner][ceil(k/64)],          */
/*                      plane i holds bit i of every value (dense layer:      */
/*                      inner = 1; NHWC image: outer = B, inner = H*W, k = C, */
/*                      so that each plane is itself a packed NHWC image).    */
/*   row_sums (load time): wsum int32 [N], wsum[n] = sum_k w[n][k] over the K */
/*                      true values of row n of packed weights W              */
/*                      [N][row_words] (for filters [L2][kh][kw][Cw]:         */
/*                      row_words = kh*kw*Cw, K = kh*kw*C; tail bits are 0).  */
/*   bitplane_combine:  d int32 [outer][8][inner][N], the esp_bgemm/esp_bconv */
/*                      results of the 8 planes (a 0 bit counting as -1) ->   */
/*                      y int32 [outer][inner][N] =                           */
/*                      (sum_i 2^i d_i + 255 * wsum) / 2.                     */
/* A pixel of value 0 is -1 in every plane, i.e. the -1 border of esp_bconv   */
/* IS zero padding of the image.  k < 2^22.                                   */
/* ------------------------------------------------------------------------- */
int esp_bitplane_pack_u8(const uint8_t *x, uint64_t *planes, int64_t outer, int64_t inner,
                         int64_t k, esp_stream stream);

int esp_row_sums(const uint64_t *W, int32_t *wsum, int64_t N, int64_t row_words, int64_t K,
                 esp_stream stream);

int esp_bitplane_combine(const int32_t *d, const int32_t *wsum, int32_t *y, int64_t outer,
                         int64_t inner, int64_t N, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* Dense layer on 8-bit inputs in one call (Sec. 4.3, Eq. 3), on the matrix    */
/* cores: the binary product of the 8 bit-planes of every input row with W and */
/* their weighted combination, which happens in the product's epilogue (the    */
/* eight partial results never reach memory).                                  */
/*   planes uint64 [rows][8][ceil(K/64)]  (esp_bitplane_pack_u8 with inner = 1) */
/*   W      uint64 [N][ceil(K/64)], wsum int32 [N] (esp_row_sums)              */
/*   y      int32 [rows][N] = sum_k x[r][k] * w[n][k]           (optional)     */
/*   bits   uint64 [rows][ceil(N/64)], bit n = (y >= thr[n]) XOR flipbit(n),   */
/*          thr / flip as from esp_bn_fold                      (optional)     */
/* At least one of y and bits.  Identical to esp_bgemm on the planes, then     */
/* esp_bitplane_combine, then esp_bn_sign_pack.  K < 2^21.                     */
/* ------------------------------------------------------------------------- */
int esp_bitplane_dense(const uint64_t *planes, const uint64_t *W, const int32_t *wsum,
                       const int32_t *thr, const uint64_t *flip, uint64_t *bits, int32_t *y,
                       int64_t rows, int64_t N, int64_t K, esp_stream stream);

/* ------------------------------------------------------------------------- */
/* Measurement aid: the in-register ceiling of the inner loop of Eq. 2 (Sec.  */
/* 4.2, with XOR for XNOR).  Launches `blocks` blocks of 256 lanes; every lane */
/* runs `iters` rounds of an 8 x 8 register block on values that stay in        */
/* registers (no memory traffic besides one final store per lane).  mode:       */
/*   ESP_PROBE_PAIR           v_xor_b32 + accumulating v_bcnt_u32_b32 pairs in  */
/*                            the product kernel's instruction pattern; *work = */
/*                            binary operations of the launch (64 per pair), so */
/*                            work / time compares with esp_bgemm's 2*M*N*K / t */
/*   ESP_PROBE_XOR_ONLY       two dependent v_xor_b32 per slot                  */
/*   ESP_PROBE_POPCOUNT_ONLY  two dependent v_bcnt_u32_b32 per slot             */
/*                            *work = lane instructions of the launch (64 lanes */
/*                            per wave instruction): the rate each instruction  */
/*                            sustains alone, from which the peak of the pair   */
/*                            follows as 64 / (1/xor_rate + 1/popcount_rate).   */
/* sink (device, uint32 [blocks * 256]) receives each lane's counter sum; work  */
/* is HOST memory.  blocks, iters in [1, 2^20]; another mode: ESP_EINVAL.       */
/* ------------------------------------------------------------------------- */
enum esp_probe_mode { ESP_PROBE_PAIR = 0, ESP_PROBE_XOR_ONLY = 1, ESP_PROBE_POPCOUNT_ONLY = 2 };

int esp_xor_popcount_probe(uint32_t *sink, int blocks, int iters, int mode, int64_t *work, esp_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* ESPRESSO_HIP_H */
