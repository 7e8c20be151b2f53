// Device-resident view of a linear model, passed by value to the kernel.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace linear_impl {

struct LinDev {
    const double *weight;  // [n_features rounded up to a multiple of 32][kp]: float64, zero-padded
    const double *bias;    // [kp]
    int32_t n_features, n_outputs, kp;
    int32_t transform, output;
};

// Column counts the kernel is instantiated for; a model uses the smallest one >= n_outputs.
int padded_outputs(int n_outputs);

hipError_t launch_linear(const LinDev &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                         hipStream_t stream);

}  // namespace linear_impl
