/*
 * CPU oracle for tree-ensemble inference.  TEST INFRASTRUCTURE ONLY: the product path never
 * links, loads or calls this file; only the tests, the smoke check and the bench's
 * cpu_baseline leg do.  It shares no code, header or table with the GPU path.
 *
 * What it computes is the plain definition the paper's operator representation must
 * reproduce: a decision tree is a chain of "compare one feature with a threshold, pick the
 * next node" steps that ends in a leaf (Section 3.1.2, the scalar operator graph of the
 * decision tree: assignments F_j -> x_i, comparisons x_i vs T_i, conditionals choose the
 * next node; Table 2: Output = the leaf node each sample reaches).  Ensembles (the tree
 * models listed in Table 4) reduce leaf payloads over trees; the paper gives no formula for
 * that step, so the usual one is written out: per output column, sum (or mean) of the
 * leaf values of the trees that feed the column, plus a base score, then an optional
 * monotone transform; labels are taken on the untransformed sums (Section 4.3.3: a
 * monotone operator in front of an indices operator changes nothing).
 *
 * Conventions fixed here (each is a reading of a point the paper leaves open):
 *   - a row goes LEFT iff x[feature] <= threshold, both float32, IEEE ordered compare;
 *     a NaN feature therefore goes RIGHT;
 *   - sums are accumulated in double, trees in ascending index, one rounding to float32;
 *   - MEAN divides a column's sum by the number of trees that feed that column; a column no
 *     tree feeds has an empty sum, which adds nothing to its base score;
 *   - sigmoid / softmax are evaluated in double from the unrounded value;
 *   - label, K >= 2: the smallest column index that attains the maximum unrounded raw value;
 *     K == 1: raw > 0.5 without transform, raw > 0 under sigmoid (the same decision, taken
 *     before the monotone transform).
 *
 * Everything walks the caller's node arrays as given: no renumbering, no packing.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_SUM = 0, ORACLE_MEAN = 1 };
enum { ORACLE_NONE = 0, ORACLE_SIGMOID = 1, ORACLE_SOFTMAX = 2 };

typedef struct {
    int32_t n_trees, n_features, n_outputs, leaf_width;
    const int64_t *tree_offset;
    const int32_t *feature;
    const float *threshold;
    const int32_t *left, *right;
    const float *leaf_value;
    const int32_t *tree_output; /* may be NULL: every scalar-leaf tree feeds column 0 */
    int32_t aggregate;
    const float *base_score; /* may be NULL: zeros */
    int32_t transform;
} oracle_model;

typedef struct {
    const oracle_model *m;
    const float *X;
    int64_t row_begin, row_end;
    float *scores;         /* [n_rows * K] or NULL */
    int32_t *labels;       /* [n_rows] or NULL */
    int32_t *leaf_node_id; /* [n_rows * n_trees] or NULL */
    double *raw_out;       /* [n_rows * K] or NULL: unrounded per-column value before transform */
    const double *col_trees;
} oracle_job;

/* Section 3.1.2: follow compare-and-branch steps from the root until a leaf is reached. */
static int32_t reach_leaf(const oracle_model *m, int32_t t, const float *x)
{
    const int64_t base = m->tree_offset[t];
    int32_t n = 0;
    while (m->feature[base + n] >= 0) {
        const float v = x[m->feature[base + n]];
        n = (v <= m->threshold[base + n]) ? m->left[base + n] : m->right[base + n];
    }
    return n;
}

static void *run_rows(void *arg)
{
    oracle_job *j = (oracle_job *)arg;
    const oracle_model *m = j->m;
    const int32_t K = m->n_outputs, W = m->leaf_width, T = m->n_trees, F = m->n_features;
    double *acc = (double *)malloc(sizeof(double) * (size_t)K);
    double *tr = (double *)malloc(sizeof(double) * (size_t)K);
    for (int64_t r = j->row_begin; r < j->row_end; ++r) {
        const float *x = j->X + r * F;
        for (int32_t k = 0; k < K; ++k) acc[k] = 0.0;
        for (int32_t t = 0; t < T; ++t) {
            const int32_t leaf = reach_leaf(m, t, x);
            if (j->leaf_node_id) j->leaf_node_id[r * T + t] = leaf;
            const float *val = m->leaf_value + (m->tree_offset[t] + leaf) * W;
            if (W == 1) {
                const int32_t k = m->tree_output ? m->tree_output[t] : 0;
                acc[k] += (double)val[0];
            } else {
                for (int32_t k = 0; k < K; ++k) acc[k] += (double)val[k];
            }
        }
        for (int32_t k = 0; k < K; ++k) {
            double s = acc[k];
            if (m->aggregate == ORACLE_MEAN && j->col_trees[k] > 0.0) s = s / j->col_trees[k];
            acc[k] = (m->base_score ? (double)m->base_score[k] : 0.0) + s;
            if (j->raw_out) j->raw_out[r * K + k] = acc[k];
        }
        /* labels come from the untransformed values (Section 4.3.3) */
        if (j->labels) {
            int32_t lab;
            if (K == 1) {
                lab = (m->transform == ORACLE_SIGMOID) ? (acc[0] > 0.0) : (acc[0] > 0.5);
            } else {
                lab = 0;
                for (int32_t k = 1; k < K; ++k)
                    if (acc[k] > acc[lab]) lab = k;
            }
            j->labels[r] = lab;
        }
        if (j->scores) {
            if (m->transform == ORACLE_SIGMOID) {
                for (int32_t k = 0; k < K; ++k) tr[k] = 1.0 / (1.0 + exp(-acc[k]));
            } else if (m->transform == ORACLE_SOFTMAX) {
                double mx = acc[0], z = 0.0;
                for (int32_t k = 1; k < K; ++k)
                    if (acc[k] > mx) mx = acc[k];
                for (int32_t k = 0; k < K; ++k) {
                    tr[k] = exp(acc[k] - mx);
                    z += tr[k];
                }
                for (int32_t k = 0; k < K; ++k) tr[k] = tr[k] / z;
            } else {
                for (int32_t k = 0; k < K; ++k) tr[k] = acc[k];
            }
            for (int32_t k = 0; k < K; ++k) j->scores[r * K + k] = (float)tr[k];
        }
    }
    free(acc);
    free(tr);
    return NULL;
}

/*
 * All pointers are host memory.  Returns 0, or -1 on a null/invalid argument.
 * Rows are split into contiguous blocks over n_threads POSIX threads; the result does not
 * depend on n_threads because rows are independent.
 */
int oracle_predict(int32_t n_trees, int32_t n_features, int32_t n_outputs, int32_t leaf_width,
                   const int64_t *tree_offset, const int32_t *feature, const float *threshold,
                   const int32_t *left, const int32_t *right, const float *leaf_value,
                   const int32_t *tree_output, int32_t aggregate, const float *base_score,
                   int32_t transform, const float *X, int64_t n_rows, float *scores,
                   int32_t *labels, int32_t *leaf_node_id, double *raw_out, int32_t n_threads)
{
    if (n_trees < 0 || n_features <= 0 || n_outputs <= 0 || n_rows < 0) return -1;
    if (leaf_width != 1 && leaf_width != n_outputs) return -1;
    if (n_trees > 0 && (!tree_offset || !feature || !threshold || !left || !right || !leaf_value))
        return -1;
    if (n_rows > 0 && !X) return -1;
    if (n_threads < 1) n_threads = 1;
    if ((int64_t)n_threads > n_rows) n_threads = n_rows > 0 ? (int32_t)n_rows : 1;

    oracle_model m = {n_trees, n_features, n_outputs, leaf_width, tree_offset, feature,
                      threshold, left,       right,     leaf_value, tree_output, aggregate,
                      base_score, transform};
    double *col_trees = (double *)calloc((size_t)n_outputs, sizeof(double));
    for (int32_t t = 0; t < n_trees; ++t) {
        if (leaf_width == 1) {
            const int32_t k = tree_output ? tree_output[t] : 0;
            if (k < 0 || k >= n_outputs) {
                free(col_trees);
                return -1;
            }
            col_trees[k] += 1.0;
        } else {
            for (int32_t k = 0; k < n_outputs; ++k) col_trees[k] += 1.0;
        }
    }

    oracle_job *jobs = (oracle_job *)calloc((size_t)n_threads, sizeof(oracle_job));
    pthread_t *tid = (pthread_t *)calloc((size_t)n_threads, sizeof(pthread_t));
    const int64_t per = (n_rows + n_threads - 1) / n_threads;
    for (int32_t i = 0; i < n_threads; ++i) {
        int64_t b = per * i, e = b + per;
        if (b > n_rows) b = n_rows;
        if (e > n_rows) e = n_rows;
        jobs[i] = (oracle_job){&m, X, b, e, scores, labels, leaf_node_id, raw_out, col_trees};
    }
    if (n_threads == 1) {
        run_rows(&jobs[0]);
    } else {
        for (int32_t i = 0; i < n_threads; ++i) pthread_create(&tid[i], NULL, run_rows, &jobs[i]);
        for (int32_t i = 0; i < n_threads; ++i) pthread_join(tid[i], NULL);
    }
    free(jobs);
    free(tid);
    free(col_trees);
    return 0;
}
