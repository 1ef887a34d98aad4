// Bit-packing kernels (arXiv 1705.07175): sign + pack of float rows (Eq. 1, Sec. 4.2),
// batch-norm threshold + sign + re-pack of int32 layer outputs (the bit-packing sign
// activation of Sec. 6.3 "Bit-packing"), and the same on the float outputs of the
// real-valued first layer (batch-norm folded to a float threshold on the host).
//
// All three are one pass over a [rows][C] array that emits one bit per element, so they
// share one bandwidth-oriented skeleton: a wave owns one 64-channel word column w and
// kRows consecutive rows; lane l loads element (r, 64*w + l) for each of those rows
// (every load instruction of the wave is one contiguous 256-byte segment, kRows of them
// in flight), the comparison writes its 64-lane result mask straight into a scalar
// register pair, which IS the packed word, and lanes 0..kRows-1 store one word each.
#include "esp_internal.h"

namespace esp {

constexpr int kRows = 16; // rows per wave task = independent loads in flight per lane

struct SignF32 {
    using in_t = float;
    struct Lane {};
    __device__ __forceinline__ Lane lane_state(int /*c*/, bool /*in_range*/) const { return Lane{}; }
    __device__ __forceinline__ bool bit(float x, const Lane &) const { return x >= 0.0f; }
    __device__ __forceinline__ uint64_t post(uint64_t word, int /*w*/) const { return word; }
};

struct ThresholdI32 {
    using in_t = int32_t;
    const int32_t *thr;
    const uint64_t *flip;
    struct Lane { int32_t t; };
    __device__ __forceinline__ Lane lane_state(int c, bool in_range) const
    {
        return Lane{in_range ? thr[c] : 0};
    }
    __device__ __forceinline__ bool bit(int32_t x, const Lane &s) const { return x >= s.t; }
    __device__ __forceinline__ uint64_t post(uint64_t word, int w) const { return word ^ flip[w]; }
};

struct ThresholdF32 {
    using in_t = float;
    const float *thr;
    const float *sgn;
    struct Lane { float t, s; };
    __device__ __forceinline__ Lane lane_state(int c, bool in_range) const
    {
        return in_range ? Lane{thr[c], sgn[c]} : Lane{0.0f, 1.0f};
    }
    // sgn is +1 or -1, so sgn * x is exact; NaN compares false (bit 0)
    __device__ __forceinline__ bool bit(float x, const Lane &l) const { return l.s * x >= l.t; }
    __device__ __forceinline__ uint64_t post(uint64_t word, int /*w*/) const { return word; }
};

template <class Op>
__global__ __launch_bounds__(256)
void rowbits_kernel(const typename Op::in_t *__restrict__ x, uint64_t *__restrict__ out,
                    int64_t rows, int C, int Cw, int64_t tasks, Op op)
{
    using in_t = typename Op::in_t;
    const int lane = threadIdx.x % kWave;
    const int64_t wave0 = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x / kWave);

    for (int64_t task = wave0; task < tasks; task += nwaves) {
        const int w = (int)(task % Cw);
        const int64_t r0 = (task / Cw) * kRows;
        const int c = w * 64 + lane;
        const bool in_range = c < C;
        const typename Op::Lane st = op.lane_state(c, in_range);

        in_t v[kRows];
        const in_t *p = x + r0 * C + c;
        if (r0 + kRows <= rows) {
#pragma unroll
            for (int j = 0; j < kRows; ++j)
                v[j] = in_range ? p[(int64_t)j * C] : in_t(0);
        } else {
#pragma unroll
            for (int j = 0; j < kRows; ++j)
                v[j] = (in_range && r0 + j < rows) ? p[(int64_t)j * C] : in_t(0);
        }
        uint64_t mine = 0;
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            const uint64_t word = __ballot(in_range && op.bit(v[j], st));
            if (lane == j)
                mine = word;
        }
        if (lane < kRows && r0 + lane < rows)
            out[(r0 + lane) * Cw + w] = op.post(mine, w);
    }
}

template <class Op>
static int launch_rowbits(const typename Op::in_t *x, uint64_t *out, int64_t rows, int64_t C,
                          Op op, hipStream_t stream)
{
    const int64_t Cw = ceil_div(C, 64);
    const int64_t tasks = Cw * ceil_div(rows, kRows);
    const unsigned grid = grid_for(tasks, 4);
    hipLaunchKernelGGL((rowbits_kernel<Op>), dim3(grid), dim3(256), 0, stream, x, out, rows, (int)C,
                       (int)Cw, tasks, op);
    return launch_status();
}

} // namespace esp

extern "C" int esp_pack_f32(const float *src, uint64_t *dst, int64_t rows, int64_t k, esp_stream stream)
{
    using namespace esp;
    if (rows < 0 || k <= 0)
        return ESP_EINVAL;
    if (k >= kMaxK)
        return ESP_ESHAPE;
    if (rows == 0)
        return ESP_OK;
    if (!src || !dst)
        return ESP_EINVAL;
    if (!aligned(src, 4) || !aligned(dst, 8))
        return ESP_EALIGN;
    return launch_rowbits<SignF32>(src, dst, rows, k, SignF32{}, as_stream(stream));
}

extern "C" int esp_bn_sign_pack(const int32_t *x, const int32_t *thr, const uint64_t *flip,
                                uint64_t *out, int64_t rows, int C, esp_stream stream)
{
    using namespace esp;
    if (rows < 0 || C <= 0)
        return ESP_EINVAL;
    if (rows == 0)
        return ESP_OK;
    if (!x || !thr || !flip || !out)
        return ESP_EINVAL;
    if (!aligned(x, 4) || !aligned(thr, 4) || !aligned(flip, 8) || !aligned(out, 8))
        return ESP_EALIGN;
    return launch_rowbits<ThresholdI32>(x, out, rows, C, ThresholdI32{thr, flip}, as_stream(stream));
}

extern "C" int esp_bn_sign_pack_f32(const float *x, const float *thr, const float *sgn,
                                    uint64_t *out, int64_t rows, int C, esp_stream stream)
{
    using namespace esp;
    if (rows < 0 || C <= 0)
        return ESP_EINVAL;
    if (rows == 0)
        return ESP_OK;
    if (!x || !thr || !sgn || !out)
        return ESP_EINVAL;
    if (!aligned(x, 4) || !aligned(thr, 4) || !aligned(sgn, 4) || !aligned(out, 8))
        return ESP_EALIGN;
    return launch_rowbits<ThresholdF32>(x, out, rows, C, ThresholdF32{thr, sgn}, as_stream(stream));
}
