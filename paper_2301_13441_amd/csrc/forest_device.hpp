// Device-resident view of a packed model, passed by value to the kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_model.hpp"

namespace forest_impl {

// Device tables of the register-bank program (forest_model.hpp, forest_pack.cpp).
struct BankDev {
    const uint32_t *prog;
    const uint32_t *child;
    const uint32_t *leaf;
    const BankTree *tree;
    const BankSpan *span;
    const BankBatch *batch;
    const BankPass *pass;           // [passes]
    const BankPassWave *pass_wave;  // [passes][BANK_WAVES]
    const BankTodo *todo;
    int32_t stream_base[BANK_WAVES];
    int32_t batches, max_units, enabled;
    int32_t passes;
};

struct DevModel {
    const SplitEntry *prog;
    const uint32_t *prog32;
    const ChildRef *child;
    const float *leaf_value;
    const int32_t *leaf_node;
    const TreeMeta *tree;
    const double *col_trees;
    const float *base;
    int32_t n_trees, n_features, n_outputs, leaf_width;
    int32_t aggregate, transform, output, kind;
    int32_t max_words;
    int32_t path;            // PATH_LDS / PATH_REG / PATH_RANK
    int32_t reg_nv, reg_r;   // REG family: 32 * reg_nv feature registers, reg_r rows per lane
    // RANK family
    int32_t rank_regs;
    int32_t lds_waves;  // LDS rank family: wavefronts per workgroup
    int32_t wave_tree[RANKLDS_WAVES_WIDE + 1];  // and the trees of each wave when the launch is not split
    const FeatBucket *feat_bucket;
    const int32_t *bucket_start;
    const float *thr_sorted;
    const int32_t *feat_thr_base;
    const int32_t *feat_vfirst;
    const FastLookup *fast_feat;  // [n_features] fast lookups (forest_rank_common.hpp)
    const uint16_t *fast_tab;
    // Tree splitting for small batches: with n_splits > 1 the grid's y index selects a share of
    // the trees and the kernels store raw fp64 partial sums to partial[(split * split_rows + row)
    // * n_outputs + k] instead of finishing the row; reduce_splits() finishes.  Set per launch.
    int32_t n_splits;
    int64_t split_rows;
    double *partial;
    int64_t partial_capacity;  // doubles available at `partial`
    int64_t n_entries;         // entries of the split program, all trees (padding included)
    // Rank families, split launches: the rank tiles ([tile][rank register][lane] packed f16 pairs)
    // are computed once per row tile by forest_rank_tiles_kernel instead of by every workgroup.
    uint32_t *rank_tiles;
    // LDS rank family: large batches of models it fits run the register-bank kernel
    BankDev bank;
};

// Batches below this many workgroups split the trees over several workgroups per row tile.
constexpr int64_t SPLIT_BELOW_BLOCKS = 512;
// A split launch aims at about this many workgroups in all and gives every wave whole trees of
// at least this many program entries together.
constexpr int64_t SPLIT_TARGET_BLOCKS = 1024;
constexpr int64_t SPLIT_MIN_ENTRIES_PER_WAVE = 512;
// Rows one workgroup of the model's kernel family owns, and its number of wavefronts.
int family_rows_per_block(const DevModel &m);
int family_waves_per_block(const DevModel &m);

// Device memory a split launch (small batch) needs besides the inputs and outputs: the tree
// shares' fp64 partial sums and, for the rank families, the rank tiles of the batch.
struct Workspace {
    double *partial = nullptr;
    int64_t partial_doubles = 0;
    uint32_t *rank_tiles = nullptr;
    int64_t rank_tile_words = 0;
};

// Lays a workspace out in `bytes` bytes at `base` (256-byte aligned): the rank tiles first, sized
// for `tiles` row tiles of the model, the partial sums in the rest.
Workspace carve_workspace(const DevModel &m, void *base, size_t bytes, int64_t tiles);

// Bytes of a workspace that never limits a split launch of the model.
size_t full_workspace_bytes(int rank_regs, int n_outputs);

// Enqueues one pass over `n_rows` rows on `stream`.  `scores` / `labels` / `leaf_out` may be
// null (that part is not written).  `ws` is the workspace a small batch may use (null: the trees
// are never cut into shares).  With `must_fit`, a small batch whose split launch does not fit
// `ws` is refused with hipErrorMemoryAllocation instead of being run unsplit.  Returns the launch
// error, if any.
hipError_t launch_predict(const DevModel &m, const Workspace *ws, bool must_fit, const float *X, int64_t n_rows,
                          float *scores, int32_t *labels, int32_t *leaf_out, hipStream_t stream);

// The calling device's copy of the library's static scratch array (set up by init_kernels), and
// its size in bytes; null before init_kernels has run on the device.
void *static_scratch(int device);
size_t static_scratch_bytes();

// Register-resident family (forest_kernels_reg.hip).
hipError_t init_reg_kernels(size_t lds_limit);
hipError_t launch_reg(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                      int32_t *leaf_out, hipStream_t stream);

// Rank family (forest_kernels_rank.hip).
hipError_t init_rank_kernels(size_t lds_limit);
hipError_t launch_rank(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                       int32_t *leaf_out, hipStream_t stream);

// LDS-resident rank family (forest_kernels_ranklds.hip).
hipError_t init_ranklds_kernels(size_t lds_limit);
hipError_t launch_ranklds(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                          int32_t *leaf_out, size_t lds_limit, hipStream_t stream);

// Register-bank kernel of the LDS rank family (forest_kernels_rankbank.hip).
hipError_t init_rankbank_kernels(size_t lds_limit);
hipError_t launch_rankbank(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                           int32_t *leaf_out, size_t lds_limit, hipStream_t stream);

// Sums the partial sums of a split launch over the splits and finishes every row.
hipError_t launch_reduce_splits(const DevModel &m, int64_t n_rows, float *scores, int32_t *labels,
                                hipStream_t stream);

// Threshold ranks of every 128-row tile of the batch into m.rank_tiles (rank families).
hipError_t launch_rank_tiles(const DevModel &m, const float *X, int64_t n_rows, hipStream_t stream);

// Whether the kernels' LDS working set for this model fits a compute unit (host-only check).
bool model_fits(const PackedModel &m);

// One-time per-process kernel attribute setup (dynamic LDS limits).
hipError_t init_kernels();

}  // namespace forest_impl
