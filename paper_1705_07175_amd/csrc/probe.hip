// In-register ceiling of the inner loop of the binary product (arXiv 1705.07175, Eq. 2 with
// XOR in place of XNOR): nothing but v_xor_b32 + accumulating v_bcnt_u32_b32 on values that
// never leave the register file.  It measures what the vector ALUs sustain (instruction issue
// and the clock the chip settles at under this load), i.e. the bound that the tiled product
// can approach but not pass.  A measurement aid, not a step of the forward path.
#include "esp_internal.h"

namespace esp {

constexpr int kProbeThreads = 256;
constexpr int kProbeRows = 8, kProbeCols = 8;   // the register block of the tiled kernel

// Every lane runs `iters` rounds of an 8 x 8 block of xor + popcount-accumulate pairs, in the
// instruction pattern of the tiled kernel's inner step (a scalar no-op after each pair; the
// compiler adds the one between consecutive asm statements).  The pairs are opaque to the
// optimiser (it would otherwise hoist the loop-invariant XORs), and the 64 counters are summed
// into `sink` so that the work is observable.
//
// MODE 1 and 2 issue the two instructions separately -- two dependent v_xor_b32, or two dependent
// accumulating v_bcnt_u32_b32, per slot of the same 8 x 8 register block -- which gives the rate
// each of them sustains alone: the two numbers from which the peak of the pair follows.
template <int MODE>
__global__ __launch_bounds__(kProbeThreads) void xor_popcount_probe_kernel(uint32_t *__restrict__ sink, int iters)
{
    uint32_t a[kProbeRows], b[kProbeCols], acc[kProbeRows][kProbeCols];
    const uint32_t seed = blockIdx.x * kProbeThreads + threadIdx.x;
    for (int i = 0; i < kProbeRows; ++i)
        a[i] = seed * 2654435761u + 0x9e3779b9u * (i + 1);
    for (int j = 0; j < kProbeCols; ++j)
        b[j] = seed * 40503u + 0x85ebca6bu * (j + 1);
    for (int i = 0; i < kProbeRows; ++i)
        for (int j = 0; j < kProbeCols; ++j)
            acc[i][j] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kProbeRows; ++i)
#pragma unroll
            for (int j = 0; j < kProbeCols; j += 4) {
                if (MODE == ESP_PROBE_XOR_ONLY) {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        asm volatile("v_xor_b32 %0, %1, %0\n\tv_xor_b32 %0, %2, %0"
                                     : "+v"(acc[i][j + c]) : "v"(a[i]), "v"(b[j + c]));
                    continue;
                }
                if (MODE == ESP_PROBE_POPCOUNT_ONLY) {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        asm volatile("v_bcnt_u32_b32 %0, %1, %0\n\tv_bcnt_u32_b32 %0, %2, %0"
                                     : "+v"(acc[i][j + c]) : "v"(a[i]), "v"(b[j + c]));
                    continue;
                }
                uint32_t t;
                asm volatile("v_xor_b32 %0, %5, %6\n\tv_bcnt_u32_b32 %1, %0, %1\n\ts_nop 0\n\t"
                             "v_xor_b32 %0, %5, %7\n\tv_bcnt_u32_b32 %2, %0, %2\n\ts_nop 0\n\t"
                             "v_xor_b32 %0, %5, %8\n\tv_bcnt_u32_b32 %3, %0, %3\n\ts_nop 0\n\t"
                             "v_xor_b32 %0, %5, %9\n\tv_bcnt_u32_b32 %4, %0, %4"
                             : "=&v"(t), "+v"(acc[i][j]), "+v"(acc[i][j + 1]), "+v"(acc[i][j + 2]), "+v"(acc[i][j + 3])
                             : "v"(a[i]), "v"(b[j]), "v"(b[j + 1]), "v"(b[j + 2]), "v"(b[j + 3]));
            }
    }
    uint32_t s = 0;
    for (int i = 0; i < kProbeRows; ++i)
        for (int j = 0; j < kProbeCols; ++j)
            s += acc[i][j];
    sink[(int64_t)blockIdx.x * kProbeThreads + threadIdx.x] = s;
}

} // namespace esp

extern "C" int esp_xor_popcount_probe(uint32_t *sink, int blocks, int iters, int mode, int64_t *work,
                                      esp_stream stream)
{
    using namespace esp;
    if (!sink || !work || blocks <= 0 || iters <= 0)
        return ESP_EINVAL;
    if (mode != ESP_PROBE_PAIR && mode != ESP_PROBE_XOR_ONLY && mode != ESP_PROBE_POPCOUNT_ONLY)
        return ESP_EINVAL;
    if (blocks > (1 << 20) || iters > (1 << 20))
        return ESP_ESHAPE;
    const int64_t slots = (int64_t)blocks * kProbeThreads * iters * kProbeRows * kProbeCols;
    const dim3 grid(blocks), block(kProbeThreads);
    if (mode == ESP_PROBE_PAIR) {
        // one pair = 32 binary multiply-accumulates = 64 binary operations
        *work = slots * 64;
        hipLaunchKernelGGL(xor_popcount_probe_kernel<ESP_PROBE_PAIR>, grid, block, 0, (hipStream_t)stream, sink, iters);
    } else if (mode == ESP_PROBE_XOR_ONLY) {
        *work = slots * 2;       // lane instructions
        hipLaunchKernelGGL(xor_popcount_probe_kernel<ESP_PROBE_XOR_ONLY>, grid, block, 0, (hipStream_t)stream, sink,
                           iters);
    } else {
        *work = slots * 2;
        hipLaunchKernelGGL(xor_popcount_probe_kernel<ESP_PROBE_POPCOUNT_ONLY>, grid, block, 0, (hipStream_t)stream,
                           sink, iters);
    }
    return launch_status();
}
