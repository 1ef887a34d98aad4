// Bit-packing kernels (arXiv 1705.07175): sign + pack of float rows (Eq. 1, Sec. 4.2),
// batch-norm threshold + sign + re-pack of int32 layer outputs (the bit-packing sign
// activation of Sec. 6.3 "Bit-packing"), and the same on the float outputs of the
// real-valued first layer (batch-norm folded to a float threshold on the host).
//
// All three are one pass over a [rows][C] array that emits one bit per element, so they
// share one bandwidth-oriented skeleton: lane l of a wave loads the element of bit
// position l of a word (every load instruction of the wave is one contiguous 256-byte
// segment, kRows of them in flight), the comparison writes its 64-lane result mask
// straight into a scalar register pair, which IS the packed word, and lanes 0..kRows-1
// store one word each.  Two task shapes: kRows consecutive words of the flat array when
// C is a multiple of 64 (rowbits_flat_kernel), one word column over kRows consecutive
// rows otherwise (rowbits_kernel).
#include "esp_internal.h"

namespace esp {

constexpr int kRows = 16; // words per wave task = independent loads in flight per lane

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
    int C;
    struct Lane { int32_t t; };
    __device__ __forceinline__ Lane lane_state(int c, bool in_range) const
    {
        return Lane{in_range ? thr[c] : 0};
    }
    __device__ __forceinline__ bool bit(int32_t x, const Lane &s) const { return x >= s.t; }
    __device__ __forceinline__ uint64_t post(uint64_t word, int w) const { return word ^ (flip[w] & valid_cols_mask(w, C)); }
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

// The same when C is a multiple of 64: rows are then whole words and, rows being contiguous,
// the array is one flat run of 64-value words.  A wave task is 16 consecutive words, so its 16
// loads cover 4 KB of contiguous memory and its 16 output words are one 128-byte store (the
// column-per-wave shape above walks 16 rows that lie C * 4 bytes apart and scatters 8-byte
// stores over them).  PERIODIC: Cw divides 16, so the channel of word j of a task is the same
// in every task and the per-channel state is fetched once per wave; otherwise Cw >= 16 and the
// word position inside the row is carried along (one wrap per step at most).
template <class Op, bool PERIODIC>
__global__ __launch_bounds__(256)
void rowbits_flat_kernel(const typename Op::in_t *__restrict__ x, uint64_t *__restrict__ out,
                         int Cw, int64_t words, int64_t tasks, Op op)
{
    using in_t = typename Op::in_t;
    const int lane = threadIdx.x % kWave;
    const int64_t wave0 = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x / kWave);
    typename Op::Lane fixed[PERIODIC ? kRows : 1];
    if (PERIODIC) {
#pragma unroll
        for (int j = 0; j < kRows; ++j)
            fixed[j] = op.lane_state((j % Cw) * 64 + lane, true);
    }
    int w0 = (int)((wave0 * kRows) % Cw);               // word position of the task's first word
    const int w_step = (int)((nwaves * kRows) % Cw);
    for (int64_t task = wave0; task < tasks; task += nwaves, w0 = w0 + w_step >= Cw ? w0 + w_step - Cw : w0 + w_step) {
        const int64_t g0 = task * kRows;
        const in_t *p = x + g0 * 64 + lane;
        in_t v[kRows];
        if (g0 + kRows <= words) {
#pragma unroll
            for (int j = 0; j < kRows; ++j)
                v[j] = p[j * 64];
        } else {
#pragma unroll
            for (int j = 0; j < kRows; ++j)
                v[j] = g0 + j < words ? p[j * 64] : in_t(0);
        }
        uint64_t mine = 0;
#pragma unroll
        for (int j = 0; j < kRows; ++j) {
            uint64_t word;
            if (PERIODIC)
                word = __ballot(op.bit(v[j], fixed[j]));
            else
                word = __ballot(op.bit(v[j], op.lane_state((w0 + j >= Cw ? w0 + j - Cw : w0 + j) * 64 + lane, true)));
            if (lane == j)
                mine = word;
        }
        if (lane < kRows && g0 + lane < words) {
            const int wl = PERIODIC ? lane % Cw : (w0 + lane >= Cw ? w0 + lane - Cw : w0 + lane);
            out[g0 + lane] = op.post(mine, wl);
        }
    }
}

template <class Op>
static int launch_rowbits(const typename Op::in_t *x, uint64_t *out, int64_t rows, int64_t C,
                          Op op, hipStream_t stream)
{
    const int64_t Cw = ceil_div(C, 64);
    if (C % 64 == 0 && (kRows % Cw == 0 || Cw >= kRows)) {
        const int64_t words = rows * Cw;
        const int64_t tasks = ceil_div(words, kRows);
        const dim3 grid(grid_for(tasks, 4));
        if (kRows % Cw == 0)
            hipLaunchKernelGGL((rowbits_flat_kernel<Op, true>), grid, dim3(256), 0, stream, x, out, (int)Cw, words,
                               tasks, op);
        else
            hipLaunchKernelGGL((rowbits_flat_kernel<Op, false>), grid, dim3(256), 0, stream, x, out, (int)Cw, words,
                               tasks, op);
        return launch_status();
    }
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
    return launch_rowbits<ThresholdI32>(x, out, rows, C, ThresholdI32{thr, flip, C}, as_stream(stream));
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
