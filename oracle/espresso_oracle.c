/*
 * espresso_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, obviously correct CPU definitions of what the binary-network
 * forward path of Espresso (arXiv 1705.07175) computes.  Everything here works
 * on UNPACKED values: +1/-1 held one per int8_t, integer sums in int32_t, all
 * floating point in double.  There is no blocking, no fusion, no popcount and
 * no packed arithmetic: each function is the textbook definition written out,
 * so that it can be checked against the paper by eye.
 *
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg may
 * call this file.  It shares no code with the GPU library and includes none of
 * its headers.
 *
 * Layout conventions (Sec. 5.1 "Tensors"): a tensor M x N x L is row-major
 * with interleaved channels, element (m,n,l) at (m*N+n)*L+l.  A batch index is
 * prepended as the slowest dimension (the paper runs batch 1).  Dense weights
 * hold one neuron per row, [N][K] (Sec. 5.1, last paragraph).
 *
 * Build:  gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC \
 *             -o libespresso_oracle.so espresso_oracle.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of host threads used by the loops over independent output rows.
 * 1 unless the caller asks for more; the arithmetic does not depend on it. */
static int g_threads = 1;

void orc_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int orc_get_threads(void) { return g_threads; }

int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------ */
/* Eq. 1: sign activation.  x >= 0 gives +1, everything else (negatives and  */
/* NaN, for which the comparison is false) gives -1.  -0.0 >= 0 is true.     */
/* ------------------------------------------------------------------------ */
void orc_sign_f32(const float *x, int8_t *s, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        s[i] = (x[i] >= 0.0f) ? (int8_t)1 : (int8_t)-1;
}

void orc_sign_f64(const double *x, int8_t *s, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        s[i] = (x[i] >= 0.0) ? (int8_t)1 : (int8_t)-1;
}

/* ------------------------------------------------------------------------ */
/* Sec. 4.1 encoding (-1 -> bit 0, +1 -> bit 1) and Sec. 4.2 / 5.1 packing   */
/* into 64-bit words along the last dimension.  Element k of a row goes to   */
/* word k/64, bit k%64, least significant bit first; unused tail bits of the */
/* last word are 0.  These two helpers exist only so that packed GPU buffers */
/* can be compared with unpacked oracle results.                             */
/* ------------------------------------------------------------------------ */
void orc_pm1_to_words(const int8_t *s, uint64_t *w, int64_t rows, int64_t k)
{
    const int64_t kw = (k + 63) / 64;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t j = 0; j < kw; ++j)
            w[r * kw + j] = 0;
        for (int64_t i = 0; i < k; ++i)
            if (s[r * k + i] > 0)
                w[r * kw + i / 64] |= ((uint64_t)1) << (i % 64);
    }
}

void orc_words_to_pm1(const uint64_t *w, int8_t *s, int64_t rows, int64_t k)
{
    const int64_t kw = (k + 63) / 64;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t i = 0; i < k; ++i)
            s[r * k + i] = ((w[r * kw + i / 64] >> (i % 64)) & 1u) ? (int8_t)1 : (int8_t)-1;
}

/* Number of positions at which two packed rows differ, counted one bit at a
 * time.  Used by the tests for the identity behind Eq. 2:
 *   a.b = K - 2 * (number of mismatching positions). */
int64_t orc_mismatches_words(const uint64_t *a, const uint64_t *b, int64_t kw)
{
    int64_t d = 0;
    for (int64_t j = 0; j < kw; ++j)
        for (int bit = 0; bit < 64; ++bit) {
            int ba = (int)((a[j] >> bit) & 1u);
            int bb = (int)((b[j] >> bit) & 1u);
            if (ba != bb)
                ++d;
        }
    return d;
}

/* ------------------------------------------------------------------------ */
/* Binary dense layer / binary matrix product (Sec. 4.2, the quantity Eq. 2  */
/* evaluates): C[m][n] = sum_k a[m][k] * b[n][k] on +-1 values.              */
/* ------------------------------------------------------------------------ */
void orc_dense_pm1(const int8_t *a, const int8_t *b, int32_t *c,
                   int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)a[m * K + k] * (int32_t)b[n * K + k];
            c[m * N + n] = acc;
        }
}

/* ------------------------------------------------------------------------ */
/* Convolution (Sec. 5.2 "Convolutional layers", Fig. 3): cross-correlation  */
/* of an NHWC tensor with L2 filters [L2][kh][kw][C]; positions outside the  */
/* image take pad_value (Sec. 5.2 "Zero-padding for convolutions": the       */
/* binary layers treat the border as -1; pad_value 0 gives ordinary zero     */
/* padding).  Output [B][H2][W2][L2], H2 = (H + 2*pad - kh)/stride + 1.      */
/* `in` may hold any small integers, which the pad-correction pin uses.      */
/* ------------------------------------------------------------------------ */
void orc_conv_pm1(const int8_t *in, const int8_t *filt, int32_t *out,
                  int64_t B, int64_t H, int64_t W, int64_t C, int64_t L2,
                  int64_t kh, int64_t kw, int64_t stride, int64_t pad, int pad_value)
{
    const int64_t H2 = (H + 2 * pad - kh) / stride + 1;
    const int64_t W2 = (W + 2 * pad - kw) / stride + 1;
#pragma omp parallel for num_threads(g_threads) schedule(static) collapse(2)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t m = 0; m < H2; ++m)
            for (int64_t n = 0; n < W2; ++n)
                for (int64_t l2 = 0; l2 < L2; ++l2) {
                    int32_t acc = 0;
                    for (int64_t dy = 0; dy < kh; ++dy)
                        for (int64_t dx = 0; dx < kw; ++dx) {
                            const int64_t y = m * stride + dy - pad;
                            const int64_t x = n * stride + dx - pad;
                            const int inside = (y >= 0 && y < H && x >= 0 && x < W);
                            for (int64_t c = 0; c < C; ++c) {
                                int32_t v = inside ? (int32_t)in[((b * H + y) * W + x) * C + c]
                                                   : (int32_t)pad_value;
                                acc += v * (int32_t)filt[((l2 * kh + dy) * kw + dx) * C + c];
                            }
                        }
                    out[((b * H2 + m) * W2 + n) * L2 + l2] = acc;
                }
}

/* Unrolling (Fig. 3): row (b*H2+m)*W2+n of the lowered matrix is the sliding
 * volume in[b][m*s-p : m*s-p+kh][n*s-p : n*s-p+kw][:] laid out tap by tap,
 * column (dy*kw+dx)*C + c; positions outside the image take pad_value. */
void orc_unroll_pm1(const int8_t *in, int8_t *low,
                    int64_t B, int64_t H, int64_t W, int64_t C,
                    int64_t kh, int64_t kw, int64_t stride, int64_t pad, int pad_value)
{
    const int64_t H2 = (H + 2 * pad - kh) / stride + 1;
    const int64_t W2 = (W + 2 * pad - kw) / stride + 1;
    const int64_t K = kh * kw * C;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t m = 0; m < H2; ++m)
            for (int64_t n = 0; n < W2; ++n) {
                int8_t *row = low + ((b * H2 + m) * W2 + n) * K;
                for (int64_t dy = 0; dy < kh; ++dy)
                    for (int64_t dx = 0; dx < kw; ++dx) {
                        const int64_t y = m * stride + dy - pad;
                        const int64_t x = n * stride + dx - pad;
                        const int inside = (y >= 0 && y < H && x >= 0 && x < W);
                        for (int64_t c = 0; c < C; ++c)
                            row[(dy * kw + dx) * C + c] =
                                inside ? in[((b * H + y) * W + x) * C + c] : (int8_t)pad_value;
                    }
            }
}

/* ------------------------------------------------------------------------ */
/* Batch normalisation (a layer type of Sec. 5.2; the paper prints no        */
/* formula, so the standard inference form is used), per channel = last dim: */
/*   y = gamma * (x - mean) / sqrt(var + eps) + beta                          */
/* evaluated in double, left to right: d = x - mean; t = gamma * d;          */
/* s = sqrt(var + eps); y = t / s + beta.  Parameters arrive as float and    */
/* are widened first.  Compiled with -ffp-contract=off: no fused multiply-add.*/
/* ------------------------------------------------------------------------ */
double orc_bn_value(double x, float gamma, float beta, float mean, float var, float eps)
{
    const double d = x - (double)mean;
    const double t = (double)gamma * d;
    const double s = sqrt((double)var + (double)eps);
    const double q = t / s;
    return q + (double)beta;
}

void orc_bn_i32(const int32_t *x, const float *gamma, const float *beta, const float *mean,
                const float *var, float eps, double *y, int64_t rows, int64_t C)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < C; ++c)
            y[r * C + c] = orc_bn_value((double)x[r * C + c], gamma[c], beta[c], mean[c], var[c], eps);
}

void orc_bn_f64(const double *x, const float *gamma, const float *beta, const float *mean,
                const float *var, float eps, double *y, int64_t rows, int64_t C)
{
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < C; ++c)
            y[r * C + c] = orc_bn_value(x[r * C + c], gamma[c], beta[c], mean[c], var[c], eps);
}

/* ------------------------------------------------------------------------ */
/* Max-pooling (a layer type of Sec. 5.2) on +-1 values: win x win window,   */
/* given stride, no padding, output size floor((H - win)/stride) + 1.        */
/* ------------------------------------------------------------------------ */
void orc_maxpool_pm1(const int8_t *in, int8_t *out,
                     int64_t B, int64_t H, int64_t W, int64_t C, int64_t win, int64_t stride)
{
    const int64_t H2 = (H - win) / stride + 1;
    const int64_t W2 = (W - win) / stride + 1;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t m = 0; m < H2; ++m)
            for (int64_t n = 0; n < W2; ++n)
                for (int64_t c = 0; c < C; ++c) {
                    int8_t best = -128;
                    for (int64_t dy = 0; dy < win; ++dy)
                        for (int64_t dx = 0; dx < win; ++dx) {
                            int8_t v = in[((b * H + m * stride + dy) * W + n * stride + dx) * C + c];
                            if (v > best)
                                best = v;
                        }
                    out[((b * H2 + m) * W2 + n) * C + c] = best;
                }
}

/* ------------------------------------------------------------------------ */
/* Non-binary first layer (Sec. 3: the float variants of a layer): real      */
/* inputs, +-1 weights, accumulation in double.                              */
/* ------------------------------------------------------------------------ */
void orc_dense_f64(const float *x, const int8_t *w, double *y, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k)
                acc += (double)x[m * K + k] * (double)w[n * K + k];
            y[m * N + n] = acc;
        }
}

void orc_conv_f64(const float *in, const int8_t *filt, double *out,
                  int64_t B, int64_t H, int64_t W, int64_t C, int64_t L2,
                  int64_t kh, int64_t kw, int64_t stride, int64_t pad)
{
    const int64_t H2 = (H + 2 * pad - kh) / stride + 1;
    const int64_t W2 = (W + 2 * pad - kw) / stride + 1;
#pragma omp parallel for num_threads(g_threads) schedule(static) collapse(2)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t m = 0; m < H2; ++m)
            for (int64_t n = 0; n < W2; ++n)
                for (int64_t l2 = 0; l2 < L2; ++l2) {
                    double acc = 0.0;
                    for (int64_t dy = 0; dy < kh; ++dy)
                        for (int64_t dx = 0; dx < kw; ++dx) {
                            const int64_t y = m * stride + dy - pad;
                            const int64_t x = n * stride + dx - pad;
                            if (y < 0 || y >= H || x < 0 || x >= W)
                                continue; /* zero padding contributes nothing */
                            for (int64_t c = 0; c < C; ++c)
                                acc += (double)in[((b * H + y) * W + x) * C + c] *
                                       (double)filt[((l2 * kh + dy) * kw + dx) * C + c];
                        }
                    out[((b * H2 + m) * W2 + n) * L2 + l2] = acc;
                }
}

/* ------------------------------------------------------------------------ */
/* First layer on fixed-precision input (Sec. 4.3): 8-bit unsigned inputs,   */
/* +-1 weights, exact integer sums.  This is the plain product that Eq. 3    */
/* re-assembles from bit-planes; the convolution pads with the value 0.      */
/* ------------------------------------------------------------------------ */
void orc_dense_u8(const uint8_t *x, const int8_t *w, int32_t *y, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int32_t)x[m * K + k] * (int32_t)w[n * K + k];
            y[m * N + n] = acc;
        }
}

void orc_conv_u8(const uint8_t *in, const int8_t *filt, int32_t *out,
                 int64_t B, int64_t H, int64_t W, int64_t C, int64_t L2,
                 int64_t kh, int64_t kw, int64_t stride, int64_t pad)
{
    const int64_t H2 = (H + 2 * pad - kh) / stride + 1;
    const int64_t W2 = (W + 2 * pad - kw) / stride + 1;
#pragma omp parallel for num_threads(g_threads) schedule(static) collapse(2)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t m = 0; m < H2; ++m)
            for (int64_t n = 0; n < W2; ++n)
                for (int64_t l2 = 0; l2 < L2; ++l2) {
                    int32_t acc = 0;
                    for (int64_t dy = 0; dy < kh; ++dy)
                        for (int64_t dx = 0; dx < kw; ++dx) {
                            const int64_t y = m * stride + dy - pad;
                            const int64_t x = n * stride + dx - pad;
                            if (y < 0 || y >= H || x < 0 || x >= W)
                                continue; /* zero padding */
                            for (int64_t c = 0; c < C; ++c)
                                acc += (int32_t)in[((b * H + y) * W + x) * C + c] *
                                       (int32_t)filt[((l2 * kh + dy) * kw + dx) * C + c];
                        }
                    out[((b * H2 + m) * W2 + n) * L2 + l2] = acc;
                }
}
