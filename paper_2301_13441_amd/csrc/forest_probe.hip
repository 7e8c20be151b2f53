// Measurement aid (not part of the inference ABI): the rate at which this machine issues the
// packed-f16 compare instruction the rank kernels use, with nothing else in the way.  bench.py
// times it next to the forests so that the roofline's nominal peak (256 CU x 4 SIMD x 16 lanes x
// 2.4 GHz x 2 comparisons) stands beside what the chip delivers.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/forest.h"
#include "../../include/forest_testing.h"

namespace {

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_BLOCKS = 256 * 8;  // eight waves per SIMD
constexpr int PROBE_CHAINS = 16;       // independent instructions per lane and iteration

// Sixteen independent chains of v_pk_fma_f16 ... clamp per lane, in the rank kernels' operand form
// (vector register, inline constant 4.0, scalar register read for both halves).
__global__ __launch_bounds__(PROBE_THREADS) void compare_rate_kernel(int iterations, uint32_t entry, uint32_t *sink)
{
    uint32_t a[PROBE_CHAINS];
#pragma unroll
    for (int k = 0; k < PROBE_CHAINS; ++k) a[k] = 0x3c003c00u + threadIdx.x + k;
    for (int i = 0; i < iterations; ++i) {
#pragma unroll
        for (int k = 0; k < PROBE_CHAINS; ++k)
            asm volatile("v_pk_fma_f16 %0, %0, 4.0, %1 op_sel:[0,0,1] op_sel_hi:[1,0,1] clamp" : "+v"(a[k]) : "s"(entry));
    }
    uint32_t all = 0;
#pragma unroll
    for (int k = 0; k < PROBE_CHAINS; ++k) all ^= a[k];
    if (all == 0x12345678u) sink[0] = all;  // never true for clamped values; keeps the chains alive
}

}  // namespace

extern "C" int forest_probe_compare_rate(int32_t iterations, void *stream, uint32_t *device_word, int64_t *comparisons)
{
    if (iterations < 1 || iterations > (1 << 24) || !device_word || !comparisons) return FOREST_EINVAL;
    hipLaunchKernelGGL(compare_rate_kernel, dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, static_cast<hipStream_t>(stream),
                       iterations, 0xbc00bc00u, device_word);
    if (hipGetLastError() != hipSuccess) return FOREST_EHIP;
    *comparisons = static_cast<int64_t>(PROBE_BLOCKS) * PROBE_THREADS * 2 * PROBE_CHAINS * iterations;
    return FOREST_OK;
}
