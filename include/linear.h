/*
 * linear.h -- C ABI of the linear-model family of the MI355X (gfx950) inference library.
 *
 * The linear classifiers and regressors the paper lists (Section 3.3, Table 4:
 * LogisticRegression, SGDClassifier, RidgeClassifier, LinearRegression, LinearSVC, ...) are
 * one matmul with the weight matrix plus the bias, optionally followed by a monotone
 * transform (sigmoid, softmax) and an index operator (argmax).  Redundant elimination
 * (Section 4.3.3) drops the transform in front of the index operator: labels are taken from
 * the values before the transform.
 *
 *     raw[r][k]    = bias[k] + sum_f X[r][f] * weight[f][k]
 *     scores[r][k] = raw | sigmoid(raw) | softmax_k(raw)
 *     label[r]     = first argmax_k raw[r][k]            (n_outputs >= 2)
 *                    raw > 0 (sigmoid) / raw > 0.5 (none) (n_outputs == 1)
 *
 * Products and sums are taken in float64 and rounded to float32 once, so results do not
 * depend on the order of the sum beyond float64 rounding.  Same conventions as forest.h: all
 * functions are extern "C", take plain pointers and sizes, return 0 or a negative LINEAR_E*
 * code, never throw and never abort.
 */
#ifndef LINEAR_H_
#define LINEAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct linear_model linear_model; /* opaque, immutable after linear_load */

enum { LINEAR_TRANSFORM_NONE = 0, LINEAR_TRANSFORM_SIGMOID = 1, LINEAR_TRANSFORM_SOFTMAX = 2 };
enum { LINEAR_OUT_SCORES = 0, LINEAR_OUT_LABELS = 1, LINEAR_OUT_BOTH = 2 };

enum {
    LINEAR_OK = 0,
    LINEAR_EINVAL = -1,     /* null pointer, bad size or bad enum value */
    LINEAR_ENONFINITE = -4, /* NaN or infinite weight or bias */
    LINEAR_ENOMEM = -5,     /* host or device allocation failed */
    LINEAR_EHIP = -6,       /* a HIP runtime call failed (no device, launch error, ...) */
    LINEAR_ELIMIT = -7      /* model exceeds a documented limit */
};

#define LINEAR_MAX_FEATURES 65536 /* n_features */
#define LINEAR_MAX_OUTPUTS 32     /* n_outputs (K) */
/* Limit of one call (LINEAR_ELIMIT from the predict and size calls): */
#define LINEAR_MAX_ROWS 1000000000 /* n_rows: keeps the launch inside HIP's 2^32 threads per grid axis */

/* All pointers are HOST memory, borrowed for the duration of linear_load only. */
typedef struct linear_desc {
    int32_t n_features;  /* F >= 1 */
    int32_t n_outputs;   /* K >= 1 */
    const float *weight; /* [F * K], weight[f * K + k] */
    const float *bias;   /* [K] or NULL (zeros) */
    int32_t transform;   /* LINEAR_TRANSFORM_*; SOFTMAX needs n_outputs >= 2 */
    int32_t output;      /* LINEAR_OUT_* */
} linear_desc;

/*
 * Validates the description (before any HIP call, so malformed input is reported even
 * without a GPU), widens the weights to float64 and copies them to the current HIP device.
 * On success *out owns device memory until linear_free.  On error *out is untouched.
 * The handle belongs to the device that was current at load: linear_predict returns
 * LINEAR_EINVAL while another device is current.
 */
int linear_load(const linear_desc *desc, linear_model **out);

/* Releases host and device memory. linear_free(NULL) is a no-op. */
void linear_free(linear_model *m);

/* Bytes linear_predict writes for n_rows rows (0 <= n_rows <= LINEAR_MAX_ROWS); negative
 * LINEAR_E* on error. */
int64_t linear_out_bytes(const linear_model *m, int64_t n_rows);

/*
 * Byte offsets inside `out`: scores are float32 [n_rows * n_outputs] at *scores_offset,
 * labels int32 [n_rows] at *labels_offset; an absent part reports -1.
 */
int linear_out_layout(const linear_model *m, int64_t n_rows, int64_t *scores_offset, int64_t *labels_offset);

/*
 * One pass over a batch.
 *   X       DEVICE pointer, row-major contiguous float32 [n_rows * n_features], 4-byte aligned
 *   out     DEVICE pointer, linear_out_bytes(m, n_rows) bytes, 4-byte aligned
 *   stream  hipStream_t (NULL = default stream)
 * Asynchronous: enqueues one kernel and returns; reports launch errors only.  n_rows == 0 is
 * a successful no-op.  Allocates nothing; touches no shared state, so concurrent calls on one
 * handle from different streams are allowed.
 */
int linear_predict(const linear_model *m, const float *X, int64_t n_rows, void *out, void *stream);

const char *linear_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LINEAR_H_ */
