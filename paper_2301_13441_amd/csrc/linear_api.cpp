// C ABI of the linear-model family: validation, float64 widening, upload, launch.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <new>
#include <vector>

#include "../../include/linear.h"
#include "linear_device.hpp"

using namespace linear_impl;

struct linear_model {
    LinDev dev{};
    void *blob = nullptr;
    int32_t n_features = 0, n_outputs = 0, transform = 0, output = 0;
    int device = 0;  // the device the weights live on
};

namespace {

int check(const linear_desc &d)
{
    if (d.n_features < 1 || d.n_outputs < 1 || !d.weight) return LINEAR_EINVAL;
    if (d.n_features > LINEAR_MAX_FEATURES || d.n_outputs > LINEAR_MAX_OUTPUTS) return LINEAR_ELIMIT;
    if (d.transform < LINEAR_TRANSFORM_NONE || d.transform > LINEAR_TRANSFORM_SOFTMAX) return LINEAR_EINVAL;
    if (d.output < LINEAR_OUT_SCORES || d.output > LINEAR_OUT_BOTH) return LINEAR_EINVAL;
    if (d.transform == LINEAR_TRANSFORM_SOFTMAX && d.n_outputs < 2) return LINEAR_EINVAL;
    const int64_t n = static_cast<int64_t>(d.n_features) * d.n_outputs;
    for (int64_t i = 0; i < n; ++i)
        if (!std::isfinite(d.weight[i])) return LINEAR_ENONFINITE;
    if (d.bias)
        for (int32_t k = 0; k < d.n_outputs; ++k)
            if (!std::isfinite(d.bias[k])) return LINEAR_ENONFINITE;
    return LINEAR_OK;
}

}  // namespace

extern "C" {

int linear_load(const linear_desc *desc, linear_model **out)
{
    if (!desc || !out) return LINEAR_EINVAL;
    if (int rc = check(*desc)) return rc;
    const int F = desc->n_features, K = desc->n_outputs;
    const int kp = padded_outputs(K);
    const int f_pad = (F + 31) / 32 * 32;
    std::vector<double> host;
    linear_model *m = nullptr;
    try {
        // weights [F rounded up to whole chunks of 32][kp] (zero rows past F), then the bias [kp]
        host.assign(static_cast<size_t>(f_pad + 1) * kp, 0.0);
        m = new linear_model;
    } catch (const std::bad_alloc &) {
        return LINEAR_ENOMEM;
    }
    for (int f = 0; f < F; ++f)
        for (int k = 0; k < K; ++k) host[static_cast<size_t>(f) * kp + k] = desc->weight[static_cast<size_t>(f) * K + k];
    if (desc->bias)
        for (int k = 0; k < K; ++k) host[static_cast<size_t>(f_pad) * kp + k] = desc->bias[k];
    // Everything below needs a device.
    if (hipGetDevice(&m->device) != hipSuccess) {
        (void)hipGetLastError();
        delete m;
        return LINEAR_EHIP;
    }
    const size_t bytes = host.size() * sizeof(double);
    if (hipMalloc(&m->blob, bytes) != hipSuccess) {
        const hipError_t e = hipGetLastError();
        delete m;
        return e == hipErrorOutOfMemory ? LINEAR_ENOMEM : LINEAR_EHIP;
    }
    if (hipMemcpy(m->blob, host.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(m->blob);
        delete m;
        return LINEAR_EHIP;
    }
    m->n_features = F;
    m->n_outputs = K;
    m->transform = desc->transform;
    m->output = desc->output;
    m->dev.weight = static_cast<const double *>(m->blob);
    m->dev.bias = m->dev.weight + static_cast<size_t>(f_pad) * kp;
    m->dev.n_features = F;
    m->dev.n_outputs = K;
    m->dev.kp = kp;
    m->dev.transform = desc->transform;
    m->dev.output = desc->output;
    *out = m;
    return LINEAR_OK;
}

void linear_free(linear_model *m)
{
    if (!m) return;
    if (m->blob) (void)hipFree(m->blob);
    delete m;
}

int linear_out_layout(const linear_model *m, int64_t n_rows, int64_t *scores_offset, int64_t *labels_offset)
{
    if (!m || n_rows < 0) return LINEAR_EINVAL;
    if (n_rows > LINEAR_MAX_ROWS) return LINEAR_ELIMIT;
    const int64_t score_bytes = n_rows * m->n_outputs * static_cast<int64_t>(sizeof(float));
    int64_t so = -1, lo = -1;
    switch (m->output) {
        case LINEAR_OUT_SCORES: so = 0; break;
        case LINEAR_OUT_LABELS: lo = 0; break;
        default: so = 0; lo = score_bytes; break;
    }
    if (scores_offset) *scores_offset = so;
    if (labels_offset) *labels_offset = lo;
    return LINEAR_OK;
}

int64_t linear_out_bytes(const linear_model *m, int64_t n_rows)
{
    if (!m || n_rows < 0) return LINEAR_EINVAL;
    if (n_rows > LINEAR_MAX_ROWS) return LINEAR_ELIMIT;
    int64_t bytes = 0;
    if (m->output != LINEAR_OUT_LABELS) bytes += n_rows * m->n_outputs * static_cast<int64_t>(sizeof(float));
    if (m->output != LINEAR_OUT_SCORES) bytes += n_rows * static_cast<int64_t>(sizeof(int32_t));
    return bytes;
}

int linear_predict(const linear_model *m, const float *X, int64_t n_rows, void *out, void *stream)
{
    if (!m || n_rows < 0) return LINEAR_EINVAL;
    if (n_rows > LINEAR_MAX_ROWS) return LINEAR_ELIMIT;
    if (n_rows == 0) return LINEAR_OK;
    if (!X || !out) return LINEAR_EINVAL;
    int current = -1;
    if (hipGetDevice(&current) != hipSuccess) {
        (void)hipGetLastError();
        return LINEAR_EHIP;
    }
    if (current != m->device) return LINEAR_EINVAL;
    int64_t so = -1, lo = -1;
    (void)linear_out_layout(m, n_rows, &so, &lo);
    char *base = static_cast<char *>(out);
    float *scores = so >= 0 ? reinterpret_cast<float *>(base + so) : nullptr;
    int32_t *labels = lo >= 0 ? reinterpret_cast<int32_t *>(base + lo) : nullptr;
    const hipError_t e = launch_linear(m->dev, X, n_rows, scores, labels, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LINEAR_OK : LINEAR_EHIP;
}

const char *linear_strerror(int code)
{
    switch (code) {
        case LINEAR_OK: return "ok";
        case LINEAR_EINVAL: return "invalid argument";
        case LINEAR_ENONFINITE: return "non-finite weight or bias";
        case LINEAR_ENOMEM: return "out of memory";
        case LINEAR_EHIP: return "HIP runtime error";
        case LINEAR_ELIMIT: return "model exceeds a documented limit";
        default: return "unknown error";
    }
}

}  // extern "C"
