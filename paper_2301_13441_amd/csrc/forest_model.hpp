// Internal data model shared by the host model compiler and the kernels' launcher.
//
// The packed model is the operator representation of Table 2 in a bit-level layout:
//   * W1 (feature selector, one 1 per column) is stored as the feature index of every
//     internal node, i.e. matmul(X, W1) is a gather (Section 4.3.2, sparse operator
//     replacing in its limit: one non-zero per column);
//   * W2 is the threshold of every internal node, stored next to the feature index as one
//     8-byte "split program" entry;
//   * W3 / (C, D) -- which leaves lie left/right below which internal node -- is stored as
//     child references between level-ordered internal nodes and in-ordered leaves
//     (Section 3.1.2 numbering), which is what a lane needs to pick, from its split-outcome
//     bits, the unique leaf whose root path agrees with them;
//   * E is the leaf table in in-order.
#pragma once

#include <cstdint>
#include <vector>

#include "../../include/forest.h"
#include "../../include/forest_testing.h"

namespace forest_impl {

// Kernel families.  A forest whose trees are all full with one common depth 1..8 runs the
// register-resident kernel (kind = depth); everything else runs the generic kernel (kind 0).
constexpr int KIND_GENERIC = 0;
constexpr int FULL_MAX_DEPTH = 8;

// Kernel families (PackedModel::path).
constexpr int PATH_LDS = 0;   // features read from the LDS tile for every comparison (any model)
constexpr int PATH_REG = 1;   // full trees, float32 features in vector registers
constexpr int PATH_RANK = 2;  // full trees, features rewritten as packed f16 threshold ranks
constexpr int PATH_RANK_LDS = 3;  // any trees, packed f16 threshold ranks read from LDS

// Rank family.  Local ranks 0 .. RANK_SEG of a segment of RANK_SEG consecutive thresholds are
// stored as f16 CODES: code(q) is the q-th smallest f16 value with magnitude in [256, 16384)
// (6144 negative ones, then 6144 positive ones), so codes are strictly increasing in q, two
// different codes differ by at least 1/4, and 4 * code is finite in f16.  A node with local
// threshold index j' holds -4 * code(j'), and
//     clamp_[0,1]( fma(code(rank), 4, -4 code(j')) )          (one v_pk_fma_f16, two rows)
// is exactly 1.0 iff rank > j': the fused multiply-add rounds 4 (code(rank) - code(j')) once,
// which is 0 for equal codes and at least 1 in magnitude otherwise (overflow to +-Inf included),
// with the sign of the difference.  4.0 is an inline constant of the instruction.
constexpr int RANK_CODES = 12288;
constexpr int RANK_SEG = RANK_CODES - 1;  // thresholds one rank register covers

#if defined(__HIPCC__)
__host__ __device__
#endif
inline uint16_t rank_code_bits(int q)  // f16 bit pattern of code(q), 0 <= q < RANK_CODES
{
    return q < RANK_CODES / 2 ? static_cast<uint16_t>(0x8000u | (0x5c00u + (RANK_CODES / 2 - 1 - q)))
                              : static_cast<uint16_t>(0x5c00u + (q - RANK_CODES / 2));
}

// f16 bit pattern of -4 * code(q): sign flipped, exponent field + 2
inline uint16_t rank_entry_bits(int q)
{
    const uint16_t c = rank_code_bits(q);
    return static_cast<uint16_t>(((c ^ 0x8000u) & 0x8000u) | ((c & 0x7fffu) + (2u << 10)));
}
// Full trees of depth 4 and more on the rank path: where in a tree's outcome bit string each
// internal node sits.  The walk of these trees takes up to three levels at a time from a table
// (the 7 outcomes of a complete 3-level subtree index it, the path through the subtree comes out),
// so the bits of such a subtree must be adjacent: position 0 is empty, positions 1..7 hold levels
// 0..2 (position = heap index), then the 8 subtrees rooted at level 3 follow from position 8 on,
// one field of 2^(levels - 3) - 1 bits each (local heap order: root, its children, their
// children), in the order of their roots.  Depths 4..6: that is the whole tree (levels = depth).
// Depths 7 and 8: that is the first word, levels 0..4 (levels = 5); from position 32 on follow the
// 32 subtrees rooted at level 5, one field of 2^(depth - 5) - 1 bits each, which fill the other
// words exactly.  Returns the node's level-order ordinal (heap index - 1), or -1 for a position no
// node has.  (Depths 1..3 keep the heap order: position = heap index.)
constexpr int STAGED_MIN_DEPTH = 4, STAGED_MAX_DEPTH = 6, STAGED_TOP_MAX_DEPTH = 8;
constexpr int STAGED_FIELDS_AT = 8;  // first position of the fields of the subtrees rooted at level 3
constexpr int STAGED_DEEP_AT = 32;   // and of those rooted at level 5

#if defined(__HIPCC__)
__host__ __device__
#endif
inline int staged_position_node(int depth, int pos)
{
    int root0, q, field;  // heap index of the first subtree root, position inside the fields, field size
    if (depth > STAGED_MAX_DEPTH && pos >= STAGED_DEEP_AT) {
        root0 = 32, q = pos - STAGED_DEEP_AT, field = (1 << (depth - 5)) - 1;
        if (q >= 32 * field) return -1;
    } else {
        const int levels = depth > STAGED_MAX_DEPTH ? 5 : depth;  // levels the first fields cover
        if (pos < 1) return -1;
        if (pos < STAGED_FIELDS_AT) return pos - 1;  // heap index pos
        root0 = 8, q = pos - STAGED_FIELDS_AT, field = (1 << (levels - 3)) - 1;
        if (q >= 8 * field) return -1;
    }
    const int subtree = q / field, local = q % field + 1;  // local heap index 1 .. field
    int level = 0;
    while ((2 << level) <= local) ++level;       // level of `local` inside its subtree
    const int heap = ((root0 + subtree) << level) + (local - (1 << level));
    return heap - 1;
}

// The path (0..7, first decision in bit 2) through a complete 3-level subtree whose 7 outcome
// bits are t (bit l - 1 = outcome of the node with local heap index l; 1 = right).
#if defined(__HIPCC__)
__host__ __device__
#endif
inline int staged_path(int t)
{
    int p = 1;
    for (int l = 0; l < 3; ++l) p = p + p + ((t >> (p - 1)) & 1);
    return p - 8;
}

constexpr int RANK_MAX_REGS = 128;
constexpr int RANK_BUCKETS_PER_THRESHOLD = 1;  // resolution of the per-feature bucket tables
constexpr int RANK_MAX_BUCKETS = 1 << 20;      // per feature
constexpr int RANKLDS_MAX_REGS = 256;          // rank register index is 8 bits of an entry
constexpr size_t RANKLDS_MAX_LDS = 144 * 1024; // LDS budget of the LDS-resident rank kernel
constexpr int PROGRAM_PAD_ENTRIES = 96;        // readable entries after the last tree's
constexpr int RANKLDS_WAVES_WIDE = 12;         // most wavefronts per workgroup of that kernel
// Workgroup sizes the kernel is built for, in waves: 12 where two workgroups share a CU's LDS
// (6 waves per SIMD), fewer where the model's LDS need per wave is larger.
constexpr int RANKLDS_WAVE_CHOICES[] = {12, 8, 4, 2};
constexpr size_t CU_LDS_BYTES = 160 * 1024;
constexpr int RANKLDS_CHUNK_GROUPS = 8;        // that kernel walks a level in chunks of 8 groups = 64 nodes

// Rank lookup of one feature: bucket(x) = trunc((x - lo) * scale) clamped to [0, n_buckets),
// start[bucket] .. start[bucket + 1] bracket rank(x) in the feature's sorted thresholds.
struct FeatBucket {
    float lo, scale;
    int32_t n_buckets;
    int32_t start_base;  // offset of the feature's n_buckets + 1 entries in the start table
};

// The bucket of x; non-decreasing in x for every lo and scale >= 0 (float subtraction,
// multiplication and truncation are monotone), NaN goes to bucket 0.
#if defined(__HIPCC__)
__host__ __device__
#endif
inline int32_t bucket_index(float x, float lo, float scale, int32_t n_buckets)
{
    const float t = (x - lo) * scale;
    if (!(t > 0.0f)) return 0;
    if (t >= static_cast<float>(n_buckets)) return n_buckets - 1;
    return static_cast<int32_t>(t);
}

// Fast rank lookup (rank kernels; forest_rank_common.hpp).  For a feature with FAST_WINDOW ..
// FAST_MAX_THRESHOLDS distinct thresholds over a finite positive range (fast == 1):
// bucket = trunc(clamp((x - lo) * scale, 0, last_bucket)); the table entry of the bucket (16 bits,
// at byte tab_off of the table) is where a window of FAST_WINDOW thresholds begins,
// clamp(#thresholds in lower buckets - 1, 0, n - FAST_WINDOW); the rank is that plus the number
// of the window's thresholds below x wherever the window settles it (checked against the
// thresholds).  Such a feature has one rank register and all its ranks in the lower half of the
// codes.  The host compiler refines a feature's grid (2, 4, 8 .. buckets per threshold) until no
// bucket holds more than FAST_BUCKET_FILL thresholds or the table has FAST_MAX_BUCKETS entries.
constexpr int FAST_WINDOW = 8;
constexpr int FAST_MAX_THRESHOLDS = RANK_CODES / 2 - 1;
constexpr int FAST_MAX_BUCKETS = 65535;
constexpr int FAST_BUCKET_FILL = 6;

struct FastLookup {
    float lo, scale, last_bucket;
    int32_t n;         // distinct thresholds of the feature
    uint32_t tab_off;  // bytes
    uint32_t thr_off;  // byte offset of the feature's thresholds in the sorted table
    int32_t fast;
    int32_t reserved;
};

// One entry of the split program: which feature an internal node tests and its threshold.
struct SplitEntry {
    int32_t feature_slot;  // LDS family: feature index * 64; REG family: feature index;
                           // RANK family: index of the rank register
    float threshold;       // RANK family: bit pattern of the f16 pair (-j', -j'), see forest_pack.cpp
};

// Per-tree record in processing order (trees are sorted by output column, stable).
struct TreeMeta {
    int32_t prog_base;   // first split-program entry of the tree
    int32_t n_words;     // 32-bit outcome words (generic kernel)
    int32_t child_base;  // first entry of the tree in the child-reference tables
    int32_t leaf_base;   // first entry of the tree in the per-leaf tables
    int32_t root_ref;    // 0 if the root is internal, ~0 (= -1) if the root is leaf L_0
    int32_t column;      // output column of a scalar-leaf tree
    int32_t caller_tree; // index of the tree in the caller's description
    int32_t n_internal;
};

struct ChildRef {
    int32_t left, right;  // >= 0: internal ordinal (level order); < 0: ~(in-order leaf ordinal)
};

// Register-bank kernel of the LDS rank family (large batches of models it fits): a workgroup of
// BANK_WAVES waves owns BANK_ROWS rows, four per lane.  The rank registers are dealt to the waves,
// up to BANK_REGS each, and held in vector registers (two per rank register: two rows each).
// Every wave evaluates, for up to BANK_TREES trees at a time (a batch), the internal nodes that
// test one of its registers, BANK_UNIT entries of its stream at a time, and leaves their outcome
// bits in an LDS buffer all waves share (a byte per 8 nodes and row); then every lane walks one
// (row, tree) of the batch through those bits.  The ranks are computed in passes over blocks of
// BANK_PASS_FEATURES columns of X: the workgroup copies the block's part of its rows to LDS, then
// every wave looks up the registers of ITS bank that belong to the block's features.
constexpr int BANK_WAVES = 8;
constexpr int BANK_REGS = 32;
constexpr int BANK_TREES = 2;
constexpr int BANK_ROWS = 256;
constexpr int BANK_UNIT = 16;
constexpr int BANK_PASS_FEATURES = 64;
constexpr int BANK_TILE_PITCH = BANK_PASS_FEATURES + 1;  // words per row of the staged block: an odd pitch
                                                         // keeps a column's reads free of bank conflicts
constexpr size_t BANK_MAX_LDS = 72 * 1024;     // outcome bytes and child references of a batch (a launch with 80 KB did not return: not used)
constexpr int BANK_PAD_ENTRIES = 64;        // readable entries after each wave's stream

// A prologue pass: columns [feat_begin, feat_end) of X, at most BANK_PASS_FEATURES of them.
struct BankPass {
    int32_t feat_begin, feat_end;
};

// What one wave looks up in one pass: items [begin, begin + n_fast) of the to-do list take the
// fast lookup, the n_slow items after them the general one.
struct BankPassWave {
    int32_t begin, n_fast, n_slow, reserved;
};

// One rank register to look up: register `slot` of the wave's bank holds thresholds
// [first, first + len) of `feature` (one segment of the feature's sorted thresholds).
struct BankTodo {
    int32_t slot, feature, first, len;
};


// The register-bank program's walk.  A slot's word in the child table holds, for the left child
// in the low half and the right child in the high half, the byte offset (4 * slot) of the word
// the walk reads next: the child's slot, or the slot itself where the child is a leaf.  The leaf
// table holds for the same two children their in-order index among the leaves of the tree
// (0xffff for an internal child).  A tree record's root reference is the byte offset of the
// root's word, or BANK_LEAF_FLAG if the tree is a single leaf.
constexpr uint32_t BANK_LEAF_FLAG = 0x8000u;

struct BankTree {
    int32_t root_ref;     // byte offset of the root's word in the batch's child table; BANK_LEAF_FLAG: a single leaf
    int32_t leaf_base;    // index of the tree's first leaf in the per-leaf tables
    int32_t caller_tree;  // index of the tree in the caller's description
    int32_t valid;        // 0 for the record that fills a batch of one tree
};

struct BankBatch {
    int32_t slot_base;  // first entry of the batch in the child table
    int32_t n_slots;    // slots of the batch (whole units)
    int32_t steps;      // moves of the walk: internal nodes on the longest path of the batch's trees, less one
    int32_t reserved;
};

struct BankSpan {
    int32_t n_units;    // units of BANK_UNIT entries of this wave in this batch
    int32_t unit_base;  // index of the first of them in the batch's bit buffer
};

struct PackedModel {
    int32_t n_trees = 0, n_features = 0, n_outputs = 0, leaf_width = 1;
    int32_t aggregate = 0, transform = 0, output = 0;
    int32_t kind = KIND_GENERIC;
    int32_t max_depth = 0;
    int32_t max_words = 0;  // largest TreeMeta::n_words
    // register-resident kernel family: features live in 32 * reg_nv vector registers per row
    // slot, reg_r row slots per lane; the split program then stores plain feature indices
    int32_t x_in_registers = 0, reg_nv = 0, reg_r = 0;
    // which kernel family runs the model
    int32_t path = PATH_LDS;
    // rank family: X is rewritten, exactly, as per-feature threshold ranks (see forest_pack.cpp)
    int32_t rank_regs = 0;        // packed rank registers per lane (one per virtual feature)
    int32_t lds_waves = 0;        // LDS rank family: wavefronts per workgroup
    // LDS rank family: wave w of a workgroup evaluates trees wave_tree[w] .. wave_tree[w + 1]
    // (processing order) -- contiguous runs of about equal program length
    int32_t wave_tree[RANKLDS_WAVES_WIDE + 1] = {};
    std::vector<FeatBucket> feat_bucket;  // [F] bucket table of each feature
    std::vector<int32_t> bucket_start;    // per feature: #thresholds in lower buckets, n_buckets + 1 entries
    std::vector<float> thr_sorted;        // per feature: distinct thresholds ascending, concatenated
    std::vector<int32_t> feat_thr_base;   // [F + 1] offsets into thr_sorted
    std::vector<int32_t> feat_vfirst;     // [F] first rank register of the feature
    std::vector<FastLookup> fast_feat;    // [F] fast lookups
    std::vector<uint16_t> fast_tab;       // their tables
    int64_t n_internal = 0, n_leaves = 0;

    std::vector<TreeMeta> tree;      // processing order
    std::vector<SplitEntry> prog;    // evaluation order (see forest_pack.cpp); LDS and REG families
    std::vector<uint32_t> prog32;    // RANK family: (f16(-j') << 16) | rank register
    std::vector<ChildRef> child;     // [sum N_I]
    std::vector<float> leaf_value;   // E, [sum N_L * leaf_width]
    std::vector<int32_t> leaf_node;  // [sum N_L] caller's node index of each leaf
    std::vector<double> col_trees;   // [K] number of trees feeding each column
    std::vector<float> base;         // [K]

    // register-bank program (empty unless bank_enabled)
    int32_t bank_enabled = 0;
    int32_t bank_batches = 0;
    int32_t bank_max_units = 0;              // most units a batch's bit buffer holds
    int32_t bank_stream_base[BANK_WAVES] = {};  // first entry of each wave's stream in bank_prog
    std::vector<BankPass> bank_pass;          // prologue passes (blocks of columns with rank registers)
    std::vector<BankPassWave> bank_pass_wave; // [passes][BANK_WAVES]
    std::vector<BankTodo> bank_todo;          // the waves' to-do lists, pass by pass
    std::vector<uint32_t> bank_prog;         // (f16(-4 code(j')) << 16) | register index inside the bank
    std::vector<uint32_t> bank_child;        // per batch, by slot: where the walk goes next, left | right << 16
    std::vector<uint32_t> bank_leaf;         // same index: the leaves the two children are, left | right << 16
    std::vector<BankBatch> bank_batch;       // [batches]
    std::vector<BankTree> bank_tree;         // [batches * BANK_TREES], processing order
    std::vector<BankSpan> bank_span;         // [batches][BANK_WAVES]
    std::vector<int32_t> bank_reg;           // [BANK_WAVES * BANK_REGS] rank register behind each bank register

    // caller-order views used only by forest_pack_view
    std::vector<int32_t> v_n_internal, v_depth, v_is_full, v_program_groups, v_order_leaf_tree;
    std::vector<int64_t> v_node_base, v_leaf_base;
    std::vector<int32_t> v_feature, v_left, v_right, v_leaf_node;
    std::vector<float> v_threshold, v_leaf_value;
};

// LDS of one workgroup of the LDS rank kernel with `waves` wavefronts: the rank tile, one chunk
// of outcome bytes (8 groups x 2 rows x 64 lanes) per wave and the float64 partial sums, which
// reuse the front part when they can wait in registers until every wave is done.
inline size_t ranklds_lds_bytes(int rank_regs, int n_outputs, int leaf_width, int waves)
{
    const size_t regs = rank_regs > 0 ? static_cast<size_t>(rank_regs) : 1;
    const int K = n_outputs, W = leaf_width;
    const bool deferred = (W == 1 && K == 1) || (W == K && K <= 2 && W != 1);
    const size_t front = sizeof(uint32_t) * 64 * regs + static_cast<size_t>(waves) * 8 * 2 * 64;
    if (W == 1 && K > 1) {
        // scalar leaves, several columns: the trees are sorted by column, so a wave's run of trees
        // feeds consecutive columns and the workgroup has at most waves + K - 1 (wave, column)
        // sums of 128 rows; then K summed columns, and three small integers per wave
        return front + sizeof(double) * 128 * static_cast<size_t>(waves + 2 * K - 1) + 256;
    }
    const size_t sums = sizeof(double) * static_cast<size_t>(waves) * K * 128;
    return deferred ? (front > sums ? front : sums) : front + sums;
}

// LDS of one workgroup (4 waves, 64 rows) of the plain LDS family: float64 partial sums and the
// transposed X tile when it is staged.
inline size_t plain_lds_bytes(int n_features, int n_outputs, bool staged)
{
    size_t b = sizeof(double) * 4 * static_cast<size_t>(n_outputs) * 64;
    if (staged) b += sizeof(float) * static_cast<size_t>(n_features) * 64;
    return b;
}

// Validates `d` and fills `out`.  Returns FOREST_OK or a negative FOREST_E* code.
int compile_forest(const forest_desc &d, PackedModel &out);

}  // namespace forest_impl
