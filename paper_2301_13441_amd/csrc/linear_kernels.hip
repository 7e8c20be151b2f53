// Linear models on gfx950: raw = X . W + b, transform, label (Section 4.1, Table 3; the label
// comes from the values before the transform, Section 4.3.3).
//
// The path is bound by reading X once from HBM (4 F bytes per row against 2 F K flops), so the
// kernel is a streaming one.  A wavefront owns 64 consecutive rows and walks the features in
// chunks of 32: the 64 x 32 chunk is read coalesced (a half-wave covers 128 contiguous bytes
// of a row), parked in the wave's own LDS tile with an odd row stride, and then every lane
// takes its row out of the tile and accumulates its K outputs in float64 against weights that
// are wave-uniform (scalar loads).  No barriers: the four waves of a workgroup never share
// data, and LDS operations of one wave complete in order.  Products of float32 values are
// exact in float64 and vector float64 FMA runs at full rate on this chip, so the float64
// accumulation costs no bandwidth.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/linear.h"
#include "linear_device.hpp"

namespace linear_impl {
namespace {

constexpr int LANES = 64;
constexpr int LWAVES = 4;
constexpr int CHUNK = 32;              // features per pass
constexpr int STRIDE = CHUNK + 1;      // odd row stride of the LDS tile: conflict-free column reads

template <int KP>
__global__ __launch_bounds__(LANES *LWAVES) void linear_kernel(LinDev m, const float *__restrict__ X,
                                                                int64_t n_rows, float *scores, int32_t *labels)
{
    __shared__ float tile[LWAVES][LANES * STRIDE];
    const int lane = threadIdx.x & (LANES - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float *xs = tile[wave];
    const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * LWAVES + wave) * LANES;
    if (row0 >= n_rows) return;  // wave-uniform
    const int F = m.n_features;
    const int64_t left = n_rows - row0;
    const int rows_here = left < LANES ? static_cast<int>(left) : LANES;
    const float *__restrict__ src = X + row0 * F;

    double acc[KP];
#pragma unroll
    for (int k = 0; k < KP; ++k) acc[k] = m.bias[k];

    for (int c0 = 0; c0 < F; c0 += CHUNK) {
        const int fc = F - c0 < CHUNK ? F - c0 : CHUNK;
        // element e of the chunk: row e / 32, column e % 32
#pragma unroll 8
        for (int i = 0; i < CHUNK; ++i) {
            const int r = 2 * i + (lane >> 5), c = lane & (CHUNK - 1);
            const bool in = r < rows_here && c < fc;
            xs[r * STRIDE + c] = in ? src[static_cast<int64_t>(r) * F + c0 + c] : 0.0f;
        }
        const double *__restrict__ w = m.weight + static_cast<int64_t>(c0) * KP;
        for (int c = 0; c < fc; ++c) {
            const double x = static_cast<double>(xs[lane * STRIDE + c]);
#pragma unroll
            for (int k = 0; k < KP; ++k) acc[k] = __builtin_fma(x, w[c * KP + k], acc[k]);
        }
    }

    if (lane >= rows_here) return;
    const int64_t row = row0 + lane;
    const int K = m.n_outputs;
    double best = acc[0];
    int best_k = 0;
#pragma unroll
    for (int k = 1; k < KP; ++k)
        if (k < K && acc[k] > best) {
            best = acc[k];
            best_k = k;
        }
    if (labels) {
        int lab = best_k;
        if (K == 1) lab = (m.transform == LINEAR_TRANSFORM_SIGMOID) ? (best > 0.0) : (best > 0.5);
        labels[row] = lab;
    }
    if (!scores) return;
    float *dst = scores + row * K;
    if (m.transform == LINEAR_TRANSFORM_SOFTMAX) {
        double z = 0.0;
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) {
                acc[k] = exp(acc[k] - best);
                z += acc[k];
            }
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) dst[k] = static_cast<float>(acc[k] / z);
    } else if (m.transform == LINEAR_TRANSFORM_SIGMOID) {
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) dst[k] = static_cast<float>(1.0 / (1.0 + exp(-acc[k])));
    } else {
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) dst[k] = static_cast<float>(acc[k]);
    }
}

using LinearFn = void (*)(LinDev, const float *, int64_t, float *, int32_t *);

LinearFn pick(int kp)
{
    switch (kp) {
        case 1: return linear_kernel<1>;
        case 2: return linear_kernel<2>;
        case 3: return linear_kernel<3>;
        case 4: return linear_kernel<4>;
        case 5: return linear_kernel<5>;
        case 6: return linear_kernel<6>;
        case 8: return linear_kernel<8>;
        case 10: return linear_kernel<10>;
        case 12: return linear_kernel<12>;
        case 16: return linear_kernel<16>;
        case 24: return linear_kernel<24>;
        case 32: return linear_kernel<32>;
        default: return nullptr;
    }
}

}  // namespace

int padded_outputs(int n_outputs)
{
    static const int sizes[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32};
    for (int s : sizes)
        if (s >= n_outputs) return s;
    return 0;
}

hipError_t launch_linear(const LinDev &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                         hipStream_t stream)
{
    if (n_rows <= 0) return hipSuccess;
    LinearFn fn = pick(m.kp);
    if (!fn) return hipErrorInvalidValue;
    const int64_t n_blocks = (n_rows + LANES * LWAVES - 1) / (LANES * LWAVES);
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(static_cast<unsigned>(n_blocks)), dim3(LANES * LWAVES), 0, stream, m, X, n_rows,
                       scores, labels);
    return hipGetLastError();
}

}  // namespace linear_impl
