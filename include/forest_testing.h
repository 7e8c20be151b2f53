/*
 * forest_testing.h -- host-only views into the model compiler of the tree-ensemble library,
 * for its tests.  Not part of the inference ABI (include/forest.h): the layouts shown here are
 * internals of the packed model and may change with the kernels.  Same conventions: extern "C",
 * plain pointers and sizes, 0 or a negative FOREST_E* code, no GPU needed.
 *
 * What the views let a test check: the numbering of Section 3.1.2 (internal nodes in level order,
 * leaves in in-order), the weights of Table 2 as the packed model stores them (split features W1,
 * thresholds W2, child references standing for W3, the leaf table E), and the exact rewriting of
 * the float32 comparison as a comparison of small-integer threshold ranks (Section 4.3.1, dtype
 * rewriting, applied to the input).
 */
#ifndef FOREST_TESTING_H_
#define FOREST_TESTING_H_

#include "forest.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Host-only view of the packed model for tests of the model compiler (no GPU needed):
 * compiles `desc` exactly as forest_load does, without uploading, and evaluates nothing.
 * The arrays below are HOST memory owned by the handle, valid until forest_pack_free.
 */
struct forest_rank_bucket {
    float lo, scale;
    int32_t n_buckets, start_base;
};

typedef struct forest_packed_view {
    int32_t n_trees;
    int32_t kernel_kind;            /* common depth of a forest of full trees (1..8), else 0 */
    int32_t kernel_path;            /* as forest_info_t.kernel_path */
    int32_t rank_registers;         /* kernel_path 2: rank registers per lane (virtual features) */
    const int32_t *tree_n_internal; /* [n_trees] N_I */
    const int32_t *tree_depth;      /* [n_trees] longest path; full trees: every path */
    const int32_t *tree_is_full;    /* [n_trees] 1 if every leaf sits at tree_depth */
    const int64_t *node_base;       /* [n_trees + 1] offsets into the per-internal-node arrays */
    const int64_t *leaf_base;       /* [n_trees + 1] offsets into the per-leaf arrays */
    const int32_t *split_feature;   /* [sum N_I] level order (I_0, I_1, ...) */
    const float *split_threshold;   /* [sum N_I] */
    const int32_t *child_left;      /* [sum N_I] >= 0: internal ordinal; < 0: ~leaf ordinal */
    const int32_t *child_right;     /* [sum N_I] */
    const int32_t *leaf_node;       /* [sum N_L] caller's tree-local node index of L_j (in-order) */
    const float *leaf_value;        /* [sum N_L * leaf_width] the table E */
    /* kernel_path 2 and 3 (else NULL): the tables that turn a feature value into its threshold
     * rank.  rank_threshold[rank_threshold_base[f] .. rank_threshold_base[f + 1]) are the
     * distinct thresholds of feature f, ascending.  rank_bucket[f] = (lo, scale, n_buckets,
     * start_base): for b = min(max(trunc((x - lo) * scale), 0), n_buckets - 1), computed in
     * float32, rank_bucket_start[start_base + b] <= rank(x) <= rank_bucket_start[start_base + b + 1]. */
    const float *rank_threshold;
    const int32_t *rank_threshold_base;        /* [n_features + 1] */
    const struct forest_rank_bucket *rank_bucket; /* [n_features] */
    const int32_t *rank_bucket_start;
    /* kernel_path 3: wavefronts per workgroup, the trees of each wavefront (processing order:
     * wave w takes trees wave_tree[w] .. wave_tree[w + 1] - 1, workgroup_waves + 1 entries) and
     * the program length of every tree in that order, in groups of 8 entries; else 0 / NULL. */
    int32_t workgroup_waves;
    const int32_t *wave_tree;
    const int32_t *program_groups; /* [n_trees] */
    /* kernel_path 3, models whose large batches run the register-bank kernel (else bank_batches
     * is 0 and the pointers NULL).  The rank registers are dealt to bank_waves wavefronts,
     * bank_regs each (bank_reg[w * bank_regs + i] = rank register behind register i of wave w);
     * the trees are taken up to bank_trees at a time (a batch; which trees share one is the
     * compiler's choice).  In batch b wave
     * w evaluates bank_span[2 * (b * bank_waves + w)] units of bank_unit entries from its stream,
     * which starts at bank_prog[bank_stream_base[w]] and runs on from batch to batch; a unit's bits
     * go to unit bank_span[2 * (b * bank_waves + w) + 1] + (index of the unit) of the batch's bit
     * buffer, entry k of a unit to bit 8 * (k / 8) + 7 - k % 8.  An entry is (f16 bits of the
     * threshold's code << 16) | register index inside the bank.  Slot = bank_unit * unit + bit.
     * bank_batch[4 * b] .. + 2: first entry of batch b in bank_child and bank_leaf, its number of
     * slots, and the number of moves of its walk.  bank_child[first entry + slot] = left | right << 16:
     * where the walk goes from the node in that slot for either outcome, as 4 * slot of the child,
     * or 4 * the slot itself where the child is a leaf (0 for a slot without a node).
     * bank_leaf[first entry + slot] = left | right << 16: the in-order index, among the leaves of its
     * tree, of the leaf either child is (0xffff for an internal child; 0x80008000 for a slot without
     * a node).  The walk starts at the root, moves bank_batch[4 * b + 2] times, and the outcome of
     * the node it then stands on picks the leaf.
     * bank_tree[4 * (b * bank_trees + j)] .. + 3: 4 * slot of the root (0x8000 if the tree is a
     * single leaf), index of the tree's first leaf in order_leaf_node / order_leaf_tree, caller's
     * tree index, 1 (0 for the record that fills a batch of one tree).
     * The ranks are looked up in bank_passes passes over blocks of columns of X
     * (bank_pass[2 * p], [2 * p + 1]: first column and end).  In pass p wave w looks up items
     * [begin, begin + n_fast + n_slow) of bank_todo (bank_pass_wave[4 * (p * bank_waves + w)] .. + 2:
     * begin, n_fast, n_slow); item i is bank_todo[4 * i] .. + 3: register index inside the bank,
     * feature, first threshold and number of thresholds of the register's segment.  The first
     * n_fast items take the fast lookup (below). */
    int32_t bank_batches, bank_waves, bank_regs, bank_trees, bank_unit, bank_max_units;
    int64_t bank_prog_entries;
    const uint32_t *bank_prog;
    const int32_t *bank_stream_base; /* [bank_waves] */
    const int32_t *bank_span;        /* [bank_batches * bank_waves * 2] */
    const uint32_t *bank_child;      /* [slots of all batches] */
    const uint32_t *bank_leaf;       /* [slots of all batches] */
    const int32_t *bank_batch;       /* [bank_batches * 4] */
    const int32_t *bank_tree;        /* [bank_batches * bank_trees * 4] */
    const int32_t *bank_reg;         /* [bank_waves * bank_regs] */
    int32_t bank_passes;
    int64_t bank_todo_items;
    const int32_t *bank_pass;        /* [bank_passes * 2] */
    const int32_t *bank_pass_wave;   /* [bank_passes * bank_waves * 4] */
    const int32_t *bank_todo;        /* [bank_todo_items * 4] */
    /* kernel_path 2 and 3: the fast rank lookup of features with fast_window .. 6143 distinct
     * thresholds.  fast_feat[8 * f] .. + 7 (32-bit words): float lo, float scale, float last bucket,
     * int thresholds, byte offset of the feature's 16-bit table in fast_tab, byte offset of its
     * thresholds in rank_threshold, 1 if the feature has a fast lookup, 0.
     * bucket = trunc(clamp((x - lo) * scale, 0, last bucket)); the table entry of the bucket is the
     * index of the first of fast_window thresholds the lookup reads and counts. */
    int32_t fast_window;
    int64_t fast_tab_entries;
    const uint32_t *fast_feat;       /* [n_features * 8] */
    const uint16_t *fast_tab;        /* [fast_tab_entries] */
    const int32_t *order_leaf_node;  /* [sum N_L] caller's node index of each leaf, processing order */
    const int32_t *order_leaf_tree;  /* [sum N_L] caller's tree index of each leaf, processing order */
} forest_packed_view;

typedef struct forest_packed forest_packed;
int forest_pack(const forest_desc *desc, forest_packed **out);
int forest_pack_view(const forest_packed *p, forest_packed_view *view);
void forest_pack_free(forest_packed *p);

/*
 * Host-only view of the rank coding of kernel_path 2 and 3 (the input's dtype rewriting,
 * Section 4.3.1; no GPU needed): a rank register stores the local rank q of a row among the
 * thresholds of its segment as the f16 bit pattern *code, and a split on the segment's j-th
 * threshold carries the f16 bit pattern *entry (for q = j); the kernels take
 * clamp_[0,1](fma(code(q), 4, entry(j))), in f16 with one rounding, as the outcome bit q > j.
 * Returns the number of codes (q must be in [0, that number); one register covers one
 * threshold fewer), or FOREST_EINVAL for q out of range or a null pointer.
 */
int forest_rank_code(int32_t q, uint16_t *code, uint16_t *entry);

/*
 * Host-only view of where the rank kernels (kernel_path 2) keep the outcome bit of every internal
 * node of a full tree of depth 4 to 8 (Section 3.1.2: every internal node is evaluated; this is
 * the order their outcomes are collected in): positions 1..7 hold levels 0..2, then one field per
 * subtree rooted at level 3 follows from position 8 on, so that a table indexed by the 7 (3, 1)
 * outcomes of a complete 3- (2-, 1-) level subtree gives the path through it; at depth 7 and 8
 * this covers levels 0..4 (positions below 32) and the deeper levels keep position = heap index.
 * Stores in *node the level-order ordinal (heap index - 1) of the node at bit position `pos` of a
 * tree's 2^depth positions, -1 for a position no node has.  Returns FOREST_OK, or FOREST_EINVAL for
 * a depth outside 4..8, a position outside the tree's or a null pointer.
 */
int forest_staged_position(int32_t depth, int32_t pos, int32_t *node);

/*
 * Measurement aid: enqueues on `stream` (a hipStream_t, may be null) a kernel that does nothing
 * but issue the packed-f16 compare instruction of the rank kernels (Section 4.3.1 applied to the
 * input), `iterations` times 16 per lane on eight wavefronts per SIMD of the current device, and
 * stores the number of (row, node) comparisons that amounts to in *comparisons.  Timed by the
 * caller (events on the same stream), it gives the rate the chip delivers where the roofline
 * quotes the nominal one.  `device_word` is 4 bytes of device memory the kernel may write.
 * Returns FOREST_OK, FOREST_EINVAL (iterations outside 1 .. 2^24, null pointer) or FOREST_EHIP.
 */
int forest_probe_compare_rate(int32_t iterations, void *stream, uint32_t *device_word, int64_t *comparisons);

#ifdef __cplusplus
}
#endif
#endif /* FOREST_TESTING_H_ */
