// HIP kernels for gfx950: dense tree-ensemble inference, one lane per row.
//
// Mapping of the paper's operator graph (Fig. 2, Table 2) to a wavefront:
//   (1) matmul(X, W1)   -> gather: feature f of the wave's 64 rows, read from an LDS tile that
//                          holds X transposed ([feature][row]) and is filled by coalesced
//                          row-major reads of X;
//   (2) greater(., W2)  -> one v_cmp per (row, internal node); the threshold is wave-uniform
//                          (scalar register), the outcome is shifted into a per-lane bit word;
//   (3) matmul(., W3) + argmax -> the unique leaf whose root path agrees with the outcome
//                          bits, found by a d-step walk over the bits (the bit-level form of
//                          "first argmax of S.W3" / "T.C == D");
//   leaf gather from E, cross-tree reduction in double, LDS-staged across the waves of a
//   workgroup, then the transform; labels are taken before the transform (Section 4.3.3).
//
// This file holds the kernels that read features from the LDS tile for every comparison
// (any number of features, any tree shape), the choice of how many shares the trees of a small
// batch are cut into, and the launcher.  The other families: forest_kernels_rank.hip (packed
// f16 threshold ranks in vector registers, the headline path), forest_kernels_ranklds.hip (the
// same with the ranks in LDS, any tree shape), forest_kernels_reg.hip (float32 features in
// vector registers), forest_kernels_split.hip (what only split launches need).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"
#include "forest_kernel_common.hpp"

namespace forest_impl {
namespace {

struct Lds {
    double *acc;     // [WAVES][K][64]     per-wave partial sums
    float *xs;       // [F][64]            (staged X tile; unused when !STAGED)
};

__device__ __forceinline__ Lds carve_lds(char *smem, const DevModel &m, bool staged)
{
    Lds l;
    size_t off = 0;
    l.acc = reinterpret_cast<double *>(smem + off);
    off += sizeof(double) * WAVES * m.n_outputs * TILE;
    l.xs = reinterpret_cast<float *>(smem + off);
    return l;
}

// ---------------------------------------------------------------------------------------
// Full trees of one common depth D (1..8): outcome words live in registers, the walk is the
// implicit heap walk h -> 2h + bit(h).
// ---------------------------------------------------------------------------------------
template <int D, bool LEAVES, bool STAGED>
__global__ __launch_bounds__(BLOCK) void forest_full_kernel(DevModel m, const float *__restrict__ X,
                                                            int64_t n_rows, float *scores,
                                                            int32_t *labels, int32_t *leaf_out)
{
    extern __shared__ __align__(16) char smem[];
    const Lds lds = carve_lds(smem, m, STAGED);
    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * TILE;
    const int64_t row = row0 + lane;
    const bool valid = row < n_rows;
    const int F = m.n_features;

    if (STAGED) {
        stage_x_tile(lds.xs, X, row0, n_rows, F, TILE);
        __syncthreads();
    }
    const float *xrow = X + (valid ? row : row0) * F;  // !STAGED: direct reads of the lane's row

    Accumulator<1> accu;
    accu.init(lds.acc, wave, lane, m);

    constexpr int N_POS = 1 << D;
    constexpr int BLK = N_POS < 32 ? N_POS : 32;
    constexpr int NW = N_POS / BLK;
    const int T = m.n_trees;
    int t_begin, t_end;
    tree_range(m, wave, WAVES, t_begin, t_end);

    for (int t = t_begin; t < t_end; ++t) {
        const SplitEntry *__restrict__ p = m.prog + (static_cast<size_t>(t) << D);
        uint32_t word[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            uint32_t b = 0;
#pragma unroll
            for (int j = 0; j < BLK; ++j) {
                const SplitEntry e = p[w * BLK + j];
                const float x = STAGED ? lds.xs[e.feature_slot + lane] : xrow[e.feature_slot >> 6];
                b = b + b + (!(x <= e.threshold) ? 1u : 0u);
            }
            word[w] = b;
        }
        const int leaf = (t << D) + static_cast<int>(heap_walk<D, NW>(word));
        const TreeMeta tm = m.tree[t];
        if (LEAVES) {
            if (valid) leaf_out[row * T + tm.caller_tree] = m.leaf_node[leaf];
        } else {
            accu.begin_tree(tm.column);
            accu.add(m, 0, leaf);
        }
    }
    if (LEAVES) return;
    accu.flush();
    __syncthreads();
    if (wave == 0) finish_row(m, lds.acc, TILE, lane, row, valid, scores, labels);
}

// ---------------------------------------------------------------------------------------
// Generic trees: any shape and size.  The internal nodes are evaluated 32 at a time in level
// order; after each outcome word the lanes whose node is among its 32 follow their child
// reference.  A child comes later in level order than its parent, so one pass over the words
// ends on the leaf, and nothing but the current word is kept.
// ---------------------------------------------------------------------------------------
template <bool LEAVES, bool STAGED>
__global__ __launch_bounds__(BLOCK) void forest_generic_kernel(DevModel m, const float *__restrict__ X,
                                                               int64_t n_rows, float *scores,
                                                               int32_t *labels, int32_t *leaf_out)
{
    extern __shared__ __align__(16) char smem[];
    const Lds lds = carve_lds(smem, m, STAGED);
    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * TILE;
    const int64_t row = row0 + lane;
    const bool valid = row < n_rows;
    const int F = m.n_features;

    if (STAGED) {
        stage_x_tile(lds.xs, X, row0, n_rows, F, TILE);
        __syncthreads();
    }
    const float *xrow = X + (valid ? row : row0) * F;

    Accumulator<1> accu;
    accu.init(lds.acc, wave, lane, m);

    const int T = m.n_trees;
    int t_begin, t_end;
    tree_range(m, wave, WAVES, t_begin, t_end);

    for (int t = t_begin; t < t_end; ++t) {
        const TreeMeta tm = m.tree[t];
        const SplitEntry *__restrict__ p = m.prog + tm.prog_base;
        const ChildRef *__restrict__ ch = m.child + tm.child_base;
        int ref = tm.root_ref;  // level-order ordinal of the lane's node, or ~leaf
        for (int w = 0; w < tm.n_words; ++w) {
            uint32_t b = 0;
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const SplitEntry e = p[w * 32 + j];
                const float x = STAGED ? lds.xs[e.feature_slot + lane] : xrow[e.feature_slot >> 6];
                b = b + b + (!(x <= e.threshold) ? 1u : 0u);
            }
            // lanes standing on one of these 32 nodes move on; at the top of a tree the child
            // can be in the same word, so repeat until no lane is left in it (a validated tree
            // has no cycles: every move goes to a later ordinal or to a leaf)
            for (;;) {
                const bool here = ref >= 0 && (ref >> 5) == w;
                if (!__any(here)) break;
                if (here) {
                    const ChildRef c = ch[ref];
                    ref = ((b >> (ref & 31)) & 1u) ? c.right : c.left;
                }
            }
        }
        const int leaf = tm.leaf_base + (ref < 0 ? ~ref : 0);
        if (LEAVES) {
            if (valid) leaf_out[row * T + tm.caller_tree] = m.leaf_node[leaf];
        } else {
            accu.begin_tree(tm.column);
            accu.add(m, 0, leaf);
        }
    }
    if (LEAVES) return;
    accu.flush();
    __syncthreads();
    if (wave == 0) finish_row(m, lds.acc, TILE, lane, row, valid, scores, labels);
}

constexpr size_t LDS_LIMIT = 160 * 1024;  // LDS of one gfx950 compute unit
size_t g_lds_limit = LDS_LIMIT;            // replaced by the device's per-workgroup limit at init

static_assert(WAVES == 4 && TILE == 64, "plain_lds_bytes assumes this workgroup shape");
size_t lds_bytes(const DevModel &m, bool staged) { return plain_lds_bytes(m.n_features, m.n_outputs, staged); }

template <bool LEAVES, bool STAGED>
KernelFn pick_kernel(int kind)
{
    switch (kind) {
        case 1: return forest_full_kernel<1, LEAVES, STAGED>;
        case 2: return forest_full_kernel<2, LEAVES, STAGED>;
        case 3: return forest_full_kernel<3, LEAVES, STAGED>;
        case 4: return forest_full_kernel<4, LEAVES, STAGED>;
        case 5: return forest_full_kernel<5, LEAVES, STAGED>;
        case 6: return forest_full_kernel<6, LEAVES, STAGED>;
        case 7: return forest_full_kernel<7, LEAVES, STAGED>;
        case 8: return forest_full_kernel<8, LEAVES, STAGED>;
        default: return forest_generic_kernel<LEAVES, STAGED>;
    }
}

KernelFn pick(int kind, bool leaves, bool staged)
{
    if (leaves) return staged ? pick_kernel<true, true>(kind) : pick_kernel<true, false>(kind);
    return staged ? pick_kernel<false, true>(kind) : pick_kernel<false, false>(kind);
}

}  // namespace

// Scratch for callers that cannot allocate (forest_predict_static): one array per GPU the library
// runs on, held until the process ends.  Host code never passes the array's name to a kernel --
// on the host it is only a stand-in for the symbol -- but the device address looked up once per
// device in init_kernels.
constexpr size_t STATIC_SCRATCH_BYTES = FOREST_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int SCRATCH_MAX_DEVICES = 64;
static void *g_scratch_ptr[SCRATCH_MAX_DEVICES] = {};

void *static_scratch(int device)
{
    return device >= 0 && device < SCRATCH_MAX_DEVICES ? g_scratch_ptr[device] : nullptr;
}

size_t static_scratch_bytes() { return STATIC_SCRATCH_BYTES; }

bool model_fits(const PackedModel &m)
{
    if (m.path != PATH_LDS) return true;  // their LDS need is bounded at pack time
    return plain_lds_bytes(m.n_features, m.n_outputs, false) <= LDS_LIMIT;  // 2 KB per output column
}

hipError_t init_kernels()
{
    int dev = 0, per_block = 0;
    hipError_t e0 = hipGetDevice(&dev);
    if (e0 != hipSuccess) return e0;
    e0 = hipDeviceGetAttribute(&per_block, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e0 != hipSuccess) return e0;
    g_lds_limit = static_cast<size_t>(per_block) < LDS_LIMIT ? static_cast<size_t>(per_block) : LDS_LIMIT;
    // this device's copy of the static scratch array (each GPU holds its own, at its own address)
    if (dev < 0 || dev >= SCRATCH_MAX_DEVICES) return hipErrorInvalidDevice;
    void *scratch_ptr = nullptr;
    e0 = hipGetSymbolAddress(&scratch_ptr, HIP_SYMBOL(scratch));
    if (e0 != hipSuccess) return e0;
    g_scratch_ptr[dev] = scratch_ptr;
    for (int kind = 0; kind <= FULL_MAX_DEPTH; ++kind)
        for (int leaves = 0; leaves < 2; ++leaves)
            for (int staged = 0; staged < 2; ++staged) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick(kind, leaves, staged)),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   static_cast<int>(g_lds_limit));
                if (e != hipSuccess) return e;
            }
    if (hipError_t e = init_reg_kernels(g_lds_limit); e != hipSuccess) return e;
    if (hipError_t e = init_rank_kernels(g_lds_limit); e != hipSuccess) return e;
    if (hipError_t e = init_ranklds_kernels(g_lds_limit); e != hipSuccess) return e;
    return init_rankbank_kernels(g_lds_limit);
}

int family_rows_per_block(const DevModel &m)
{
    if (m.path == PATH_RANK || m.path == PATH_RANK_LDS) return 128;
    if (m.path == PATH_REG) return TILE * m.reg_r;
    return TILE;
}

int family_waves_per_block(const DevModel &m) { return m.path == PATH_RANK_LDS ? m.lds_waves : WAVES; }

static int64_t split_workspace_doubles(int n_outputs)
{
    // splits x rows stays below (SPLIT_TARGET_BLOCKS + SPLIT_BELOW_BLOCKS) workgroups x 128 rows
    const int64_t want = (SPLIT_TARGET_BLOCKS + SPLIT_BELOW_BLOCKS) * 128 * n_outputs;
    const int64_t cap = int64_t{4} << 20;  // 32 MB
    return want < cap ? want : cap;
}

static size_t rank_tile_bytes(int rank_regs, int64_t tiles)
{
    const size_t b = sizeof(uint32_t) * 64 * static_cast<size_t>(rank_regs > 0 ? rank_regs : 0) * static_cast<size_t>(tiles);
    return (b + 255) & ~size_t{255};
}

size_t full_workspace_bytes(int rank_regs, int n_outputs)
{
    return rank_tile_bytes(rank_regs, SPLIT_BELOW_BLOCKS) + sizeof(double) * static_cast<size_t>(split_workspace_doubles(n_outputs));
}

Workspace carve_workspace(const DevModel &m, void *base, size_t bytes, int64_t tiles)
{
    Workspace ws;
    const bool ranks = m.path == PATH_RANK || m.path == PATH_RANK_LDS;
    const size_t tile_bytes = ranks ? rank_tile_bytes(m.rank_regs, tiles) : 0;
    if (!base || tile_bytes > bytes) return ws;  // nothing fits: every launch stays unsplit
    ws.rank_tiles = static_cast<uint32_t *>(base);
    ws.rank_tile_words = static_cast<int64_t>(tile_bytes / sizeof(uint32_t));
    ws.partial = reinterpret_cast<double *>(static_cast<char *>(base) + tile_bytes);
    ws.partial_doubles = static_cast<int64_t>((bytes - tile_bytes) / sizeof(double));
    return ws;
}

namespace {

// How many shares the trees are cut into for a batch of n_rows rows (1 = no split); `fits`
// tells whether the workspace allowed the split the batch asks for.
int choose_splits(const DevModel &m, const Workspace *ws, int64_t n_rows, bool needs_sums, bool &fits)
{
    fits = true;
    const int64_t rb = family_rows_per_block(m);
    const int64_t n_blocks = (n_rows + rb - 1) / rb;
    if (n_blocks >= SPLIT_BELOW_BLOCKS) return 1;
    const int64_t per_tree = m.n_trees > 0 ? (m.n_entries + m.n_trees - 1) / m.n_trees : 1;
    const int64_t trees_per_wave = (SPLIT_MIN_ENTRIES_PER_WAVE + per_tree - 1) / (per_tree > 0 ? per_tree : 1);
    int64_t s = m.n_trees / (family_waves_per_block(m) * (trees_per_wave > 0 ? trees_per_wave : 1));
    const int64_t by_grid = (SPLIT_TARGET_BLOCKS + n_blocks - 1) / n_blocks;
    if (by_grid < s) s = by_grid;
    if (s < 2) return 1;  // the model is too small to be worth cutting
    const bool ranks = m.path == PATH_RANK || m.path == PATH_RANK_LDS;
    const int64_t tile_words = ranks ? n_blocks * m.rank_regs * 64 : 0;
    if (tile_words > (ws ? ws->rank_tile_words : 0)) {
        fits = false;
        return 1;
    }
    if (needs_sums) {
        const int64_t by_ws = (ws ? ws->partial_doubles : 0) / (n_rows * m.n_outputs);
        if (by_ws < s) s = by_ws;
        if (s < 2) {
            fits = false;
            return 1;
        }
    }
    return static_cast<int>(s);
}

}  // namespace

static hipError_t launch_family(const DevModel &m, const float *X, int64_t n_rows, float *scores,
                                int32_t *labels, int32_t *leaf_out, hipStream_t stream)
{
    if (m.path == PATH_RANK) return launch_rank(m, X, n_rows, scores, labels, leaf_out, stream);
    if (m.path == PATH_RANK_LDS) {
        // large batches of the models it fits: rank registers banked over the waves' vector registers
        if (m.n_splits == 1 && m.bank.enabled)
            return launch_rankbank(m, X, n_rows, scores, labels, leaf_out, g_lds_limit, stream);
        return launch_ranklds(m, X, n_rows, scores, labels, leaf_out, g_lds_limit, stream);
    }
    if (m.path == PATH_REG) return launch_reg(m, X, n_rows, scores, labels, leaf_out, stream);
    bool staged = true;
    if (lds_bytes(m, true) > g_lds_limit) staged = false;
    const size_t lds = lds_bytes(m, staged);
    if (lds > g_lds_limit) return hipErrorInvalidValue;
    const int64_t n_blocks = (n_rows + TILE - 1) / TILE;
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    KernelFn fn = pick(m.kind, leaf_out != nullptr, staged);
    const dim3 grid(static_cast<unsigned>(n_blocks), static_cast<unsigned>(m.n_splits));
    hipLaunchKernelGGL(fn, grid, dim3(BLOCK), lds, stream, m, X, n_rows, scores, labels, leaf_out);
    return hipGetLastError();
}

hipError_t launch_predict(const DevModel &model, const Workspace *ws, bool must_fit, const float *X, int64_t n_rows,
                          float *scores, int32_t *labels, int32_t *leaf_out, hipStream_t stream)
{
    if (n_rows <= 0) return hipSuccess;
    // Small batches: too few row tiles to fill the chip, so the trees are cut into shares as
    // well (grid y) and a second kernel sums the shares.  The leaf-id output needs no sums.
    DevModel m = model;
    const bool sums = leaf_out == nullptr;
    bool fits = true;
    m.n_splits = choose_splits(m, ws, n_rows, sums, fits);
    if (!fits && must_fit) return hipErrorMemoryAllocation;
    m.split_rows = n_rows;
    m.partial = ws ? ws->partial : nullptr;
    m.partial_capacity = ws ? ws->partial_doubles : 0;
    m.rank_tiles = ws ? ws->rank_tiles : nullptr;
    if (m.n_splits > 1 && (m.path == PATH_RANK || m.path == PATH_RANK_LDS)) {
        const hipError_t e = launch_rank_tiles(m, X, n_rows, stream);
        if (e != hipSuccess) return e;
    }
    const hipError_t e = launch_family(m, X, n_rows, scores, labels, leaf_out, stream);
    if (e != hipSuccess || m.n_splits == 1 || !sums) return e;
    return launch_reduce_splits(m, n_rows, scores, labels, stream);
}

}  // namespace forest_impl
