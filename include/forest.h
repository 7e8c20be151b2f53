/*
 * forest.h -- C ABI of the MI355X (gfx950) tree-ensemble inference library.
 *
 * The library evaluates random forests and gradient-boosted trees the way the paper's
 * operator representation does (Section 3.1.2, Table 2, Fig. 2): every internal node of
 * every tree is evaluated for every row (feature selection W1/A as a gather, element-wise
 * comparison against the thresholds W2/B), the reached leaf is resolved from the split
 * outcomes (W3 + first argmax, equivalently the signed path matrix C with path lengths D),
 * leaf payloads E are gathered and reduced across trees, and an optional monotone transform
 * is applied; labels are taken before the transform (Section 4.3.3, redundant elimination).
 *
 * All functions are extern "C", take plain pointers and sizes, return 0 or a negative
 * FOREST_E* code, never throw and never abort.
 */
#ifndef FOREST_H_
#define FOREST_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct forest forest; /* opaque; the model in it is immutable after forest_load */

enum { FOREST_AGG_SUM = 0, FOREST_AGG_MEAN = 1 };
enum { FOREST_TRANSFORM_NONE = 0, FOREST_TRANSFORM_SIGMOID = 1, FOREST_TRANSFORM_SOFTMAX = 2 };
enum { FOREST_OUT_SCORES = 0, FOREST_OUT_LABELS = 1, FOREST_OUT_BOTH = 2 };

enum {
    FOREST_OK = 0,
    FOREST_EINVAL = -1,     /* null pointer, bad size or bad enum value */
    FOREST_ETREE = -2,      /* malformed tree: child out of range, node reached twice, cycle,
                               unreachable node, empty tree */
    FOREST_EFEATURE = -3,   /* split feature >= n_features */
    FOREST_ENONFINITE = -4, /* NaN threshold (+-Inf thresholds are legal) */
    FOREST_ENOMEM = -5,     /* host or device allocation failed */
    FOREST_EHIP = -6,       /* a HIP runtime call failed (no device, launch error, ...) */
    FOREST_ELIMIT = -7      /* model exceeds a documented limit of the kernels */
};

/* Documented limits (checked at load; FOREST_ELIMIT): */
#define FOREST_MAX_FEATURES 4096  /* n_features */
#define FOREST_MAX_OUTPUTS 32     /* n_outputs (K) */
#define FOREST_MAX_DEPTH 64       /* longest root-to-leaf path, in tests */
#define FOREST_MAX_NODES (1 << 27) /* internal nodes, and leaves, summed over the trees: the split
                                      program pads levels to groups of 8 and indexes entries with int32 */
/* Limit of one call (FOREST_ELIMIT from the predict and size calls): */
#define FOREST_MAX_ROWS 1000000000 /* n_rows: keeps every launch inside HIP's 2^32 threads per grid axis */

/*
 * A forest as the caller holds it: per-node arrays, trees concatenated.  All pointers are
 * HOST memory, borrowed for the duration of forest_load only.
 *
 * Tree t owns nodes [tree_offset[t], tree_offset[t+1]); its root is the first node of the
 * range; left/right are indices local to the tree.  A node with feature < 0 is a leaf (a
 * root may be a leaf).  A row goes LEFT iff x[feature] <= threshold, as an IEEE float32
 * ordered comparison (a NaN feature goes right).
 *
 * leaf_width == 1: a leaf of tree t adds leaf_value[node] into output column
 * tree_output[t] (column 0 when tree_output is NULL).  leaf_width == n_outputs: a leaf adds
 * leaf_value[node * n_outputs + k] into every column k.
 *
 * Per column: raw = base_score[k] + (aggregate == MEAN ? sum / #trees feeding k : sum),
 * accumulated in double and rounded once; a column no tree feeds is its base score.  scores = transform(raw).  label (n_outputs >= 2)
 * = smallest k with maximal raw; n_outputs == 1: raw > 0.5 (no transform) or raw > 0 (sigmoid).
 */
typedef struct forest_desc {
    int32_t n_trees;
    int32_t n_features;
    int32_t n_outputs;         /* K >= 1 */
    int32_t leaf_width;        /* 1 or n_outputs */
    const int64_t *tree_offset; /* [n_trees + 1], non-decreasing, tree_offset[0] == 0 */
    const int32_t *feature;    /* [n_nodes] */
    const float *threshold;    /* [n_nodes] */
    const int32_t *left;       /* [n_nodes] */
    const int32_t *right;      /* [n_nodes] */
    const float *leaf_value;   /* [n_nodes * leaf_width] */
    const int32_t *tree_output; /* [n_trees] or NULL */
    int32_t aggregate;         /* FOREST_AGG_* */
    const float *base_score;   /* [n_outputs] or NULL (zeros) */
    int32_t transform;         /* FOREST_TRANSFORM_*; SOFTMAX needs n_outputs >= 2 */
    int32_t output;            /* FOREST_OUT_* */
} forest_desc;

typedef struct forest_info_t {
    int32_t n_trees, n_features, n_outputs, leaf_width;
    int64_t n_internal;    /* sum of N_I over trees = comparisons evaluated per row */
    int64_t n_leaves;      /* sum of N_L over trees */
    int32_t max_depth;     /* longest root-to-leaf path */
    int32_t kernel_kind;   /* which specialised kernel forest_predict launches (0 = generic) */
    int64_t packed_bytes;  /* device-resident size of the packed model */
    int32_t x_in_registers;     /* 1 if the kernel keeps the features in vector registers */
    int32_t kernel_path;        /* 0: features from the LDS tile; 1: float32 feature registers;
                                   2: packed f16 threshold-rank registers;
                                   3: packed f16 threshold ranks in LDS (any tree shape) */
    int32_t rows_per_workgroup; /* rows one workgroup owns */
    int64_t workspace_bytes;    /* device workspaces (all of them) the handle owns besides the packed model */
    int64_t small_batch_rows;   /* batches below this many rows also cut the trees into shares
                                   (more workgroups for few rows) and use a workspace */
    int32_t workgroup_waves;    /* wavefronts per workgroup of the kernel the model runs */
    int32_t rank_banks;         /* kernel_path 3: 1 if batches of small_batch_rows rows or more run the
                                   register-bank kernel (rank registers dealt to the wavefronts of a
                                   workgroup, whole trees evaluated before the walk) */
} forest_info_t;

/*
 * Host-side model compiler + upload (Section 3.1.2 numbering: internal nodes level order,
 * leaves in-order; Table 2 weights, stored as a packed split program, walk tables and the
 * leaf table E).  Validates the description, packs it and copies it to the current HIP
 * device.  On success *out owns device memory until forest_free.  On error *out is untouched.
 * Validation happens before any HIP call, so malformed input is reported even without a GPU.
 * The handle belongs to the device that was current at load: the predict calls return
 * FOREST_EINVAL while another device is current.
 */
int forest_load(const forest_desc *desc, forest **out);

/* Releases host and device memory. forest_free(NULL) is a no-op. */
void forest_free(forest *f);

int forest_info(const forest *f, forest_info_t *info);

/* Bytes forest_predict writes for n_rows rows (0 <= n_rows <= FOREST_MAX_ROWS); negative
 * FOREST_E* on error. */
int64_t forest_out_bytes(const forest *f, int64_t n_rows);

/*
 * Byte offsets inside `out`: scores are float32 [n_rows * n_outputs] at *scores_offset,
 * labels int32 [n_rows] at *labels_offset; an absent part reports -1.
 */
int forest_out_layout(const forest *f, int64_t n_rows, int64_t *scores_offset, int64_t *labels_offset);

/*
 * One pass of the whole path (Fig. 2 steps (1)-(3) + leaf gather + cross-tree reduction +
 * transform) over a batch.
 *   X       DEVICE pointer, row-major contiguous float32 [n_rows * n_features]
 *   out     DEVICE pointer, forest_out_bytes(f, n_rows) bytes, 4-byte aligned
 *   stream  hipStream_t (NULL = default stream)
 * Asynchronous: enqueues kernels and returns; reports launch errors only.  n_rows == 0 is a
 * successful no-op.  The caller keeps X and out alive until the stream has run the work.
 * Allocates nothing.
 * Small batches (the latency regime of Table 6): below forest_info_t.small_batch_rows rows the
 * trees are cut into shares that run in separate workgroups, their fp64 partial sums meet in a
 * workspace the handle owns and a second kernel on the same stream finishes the rows.  The handle
 * owns several such workspaces and gives every stream its own (a stream under graph capture gets
 * one for that capture), so calls on one handle may run concurrently from different streams
 * whatever their batch size; a caller that finds every workspace taken by other streams runs its
 * small batch unsplit, with the same result.
 */
int forest_predict(const forest *f, const float *X, int64_t n_rows, void *out, void *stream);

/*
 * forest_predict for callers that cannot allocate and must not depend on memory a handle
 * allocated: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same results.  The workspace of a small batch is not the handle's but a static
 * array of FOREST_STATIC_SCRATCH_BYTES in the library's device image (every GPU the library runs
 * on holds one until the process ends); the call allocates and frees nothing.  A small batch
 * whose rank tiles (ceil(n_rows / 128) * rank registers * 256 bytes for the rank kernels) and at
 * least two shares of partial sums (n_rows * n_outputs * 8 bytes each) do not fit the array is
 * refused with FOREST_ELIMIT; batches of forest_info_t.small_batch_rows rows or more use no
 * workspace and always run.  Every call on a GPU shares that GPU's array, whatever the handle:
 * calls that overlap in time on one GPU race; order them on one stream or with events.  Nothing
 * in the array needs clearing between calls (every word a call reads it has written itself).
 */
#define FOREST_STATIC_SCRATCH_BYTES (8u << 20)
int forest_predict_static(const forest *f, const float *X, int64_t n_rows, void *out, void *stream);

/*
 * Output of Table 2 ("the leaf node each sample reaches"), for tests and debugging:
 * leaf_node_id is a DEVICE pointer to int32 [n_rows * n_trees]; entry (r, t) receives the
 * caller's tree-local node index of the leaf row r reaches in tree t.
 */
int forest_predict_leaves(const forest *f, const float *X, int64_t n_rows, int32_t *leaf_node_id,
                          void *stream);

const char *forest_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* FOREST_H_ */
