// HIP kernels for gfx950: dense tree-ensemble inference, one lane per row.
//
// Mapping of the paper's operator graph (Fig. 2, Table 2) to a wavefront:
//   (1) matmul(X, W1)   -> gather: the wave reads feature f of its 64 rows from an LDS tile
//                          that holds X transposed ([feature][row]), filled by coalesced
//                          row-major reads of X;
//   (2) greater(., W2)  -> one v_cmp per (row, internal node); the threshold is wave-uniform
//                          (scalar register), the outcome is shifted into a per-lane bit word;
//   (3) matmul(., W3) + argmax -> the unique leaf whose root path agrees with the outcome
//                          bits, found by a d-step walk over the bits (the bit-level form of
//                          "first argmax of S.W3" / "T.C == D");
//   leaf gather from E, cross-tree reduction in double, LDS-staged across the waves of a
//   workgroup, then the transform; labels are taken before the transform (Section 4.3.3).
//
// A workgroup (4 wavefronts) owns a tile of 64 rows; the trees are split over its waves.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"

namespace forest_impl {
namespace {

constexpr int TILE = 64;      // rows per workgroup = lanes per wavefront
constexpr int WAVES = 4;      // wavefronts per workgroup
constexpr int BLOCK = TILE * WAVES;

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Copies rows [row0, row0 + 64) of row-major X into xs[f * 64 + r]; rows past n_rows read as 0.
__device__ __forceinline__ void stage_x_tile(float *xs, const float *X, int64_t row0, int64_t n_rows,
                                             int F)
{
    const int64_t rows_here = min(static_cast<int64_t>(TILE), n_rows - row0);
    const int n_valid = static_cast<int>(rows_here) * F;
    const float *src = X + row0 * F;
    for (int e = threadIdx.x; e < TILE * F; e += BLOCK) {
        const int r = e / F, f = e - r * F;
        xs[f * TILE + r] = (e < n_valid) ? src[e] : 0.0f;
    }
}

struct Lds {
    float *xs;       // [F][64]            (staged X tile; unused when !STAGED)
    double *acc;     // [WAVES][K][64]     per-wave partial sums
    uint32_t *bits;  // [WAVES][max_words][64] outcome words (generic kernel only)
};

__device__ __forceinline__ Lds carve_lds(char *smem, const DevModel &m, bool staged, bool generic)
{
    Lds l;
    size_t off = 0;
    l.acc = reinterpret_cast<double *>(smem + off);
    off += sizeof(double) * WAVES * m.n_outputs * TILE;
    l.xs = reinterpret_cast<float *>(smem + off);
    if (staged) off += sizeof(float) * m.n_features * TILE;
    l.bits = reinterpret_cast<uint32_t *>(smem + off);
    (void)generic;
    return l;
}

// Cross-wave reduction, aggregate, label, transform, store.  Runs on wave 0, lane = row.
__device__ __forceinline__ void finish_rows(const DevModel &m, double *acc, int64_t row, bool valid,
                                            float *scores, int32_t *labels, int lane)
{
    const int K = m.n_outputs;
    double best = 0.0;
    int best_k = 0;
    for (int k = 0; k < K; ++k) {
        double s = acc[(0 * K + k) * TILE + lane];
        for (int w = 1; w < WAVES; ++w) s += acc[(w * K + k) * TILE + lane];
        if (m.aggregate == FOREST_AGG_MEAN) s = s / m.col_trees[k];
        s = static_cast<double>(m.base[k]) + s;
        acc[k * TILE + lane] = s;  // wave 0's slice now holds the raw value
        if (k == 0 || s > best) {
            best = s;
            best_k = k;
        }
    }
    if (!valid) return;
    if (labels) {
        int lab = best_k;
        if (K == 1) lab = (m.transform == FOREST_TRANSFORM_SIGMOID) ? (best > 0.0) : (best > 0.5);
        labels[row] = lab;
    }
    if (!scores) return;
    float *dst = scores + row * K;
    if (m.transform == FOREST_TRANSFORM_SOFTMAX) {
        double z = 0.0;
        for (int k = 0; k < K; ++k) z += exp(acc[k * TILE + lane] - best);
        for (int k = 0; k < K; ++k) dst[k] = static_cast<float>(exp(acc[k * TILE + lane] - best) / z);
    } else if (m.transform == FOREST_TRANSFORM_SIGMOID) {
        for (int k = 0; k < K; ++k) dst[k] = static_cast<float>(1.0 / (1.0 + exp(-acc[k * TILE + lane])));
    } else {
        for (int k = 0; k < K; ++k) dst[k] = static_cast<float>(acc[k * TILE + lane]);
    }
}

// Adds the payload of leaf `leaf` (index into the per-leaf tables) to the wave's partial sums.
// Scalar leaves accumulate in a register per column run; vector leaves go straight to LDS.
struct Accumulator {
    double run = 0.0;
    int col = 0;
    double *mine;  // this wave's [K][64] slice
    int lane, K, W;

    __device__ __forceinline__ void init(double *acc, int wave, int lane_, const DevModel &m)
    {
        K = m.n_outputs;
        W = m.leaf_width;
        lane = lane_;
        mine = acc + static_cast<size_t>(wave) * K * TILE;
        for (int k = 0; k < K; ++k) mine[k * TILE + lane] = 0.0;
    }
    __device__ __forceinline__ void add(const DevModel &m, int column, int leaf)
    {
        if (W == 1) {
            if (column != col) {  // wave-uniform
                mine[col * TILE + lane] += run;
                run = 0.0;
                col = column;
            }
            run += static_cast<double>(m.leaf_value[leaf]);
        } else {
            const float *v = m.leaf_value + static_cast<size_t>(leaf) * K;
            for (int k = 0; k < K; ++k) mine[k * TILE + lane] += static_cast<double>(v[k]);
        }
    }
    __device__ __forceinline__ void flush()
    {
        if (W == 1) mine[col * TILE + lane] += run;
    }
};

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
    const Lds lds = carve_lds(smem, m, STAGED, false);
    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * TILE;
    const int64_t row = row0 + lane;
    const bool valid = row < n_rows;
    const int F = m.n_features;

    if (STAGED) {
        stage_x_tile(lds.xs, X, row0, n_rows, F);
        __syncthreads();
    }
    const float *xrow = X + (valid ? row : row0) * F;  // !STAGED: direct reads of the lane's row

    Accumulator accu;
    accu.init(lds.acc, wave, lane, m);

    constexpr int N_POS = 1 << D;
    constexpr int BLK = N_POS < 32 ? N_POS : 32;
    constexpr int NW = N_POS / BLK;
    const int T = m.n_trees;
    const int t_begin = static_cast<int>((static_cast<int64_t>(T) * wave) / WAVES);
    const int t_end = static_cast<int>((static_cast<int64_t>(T) * (wave + 1)) / WAVES);

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
        // walk: h = heap index of the node the row stands on
        uint32_t h = 1;
#pragma unroll
        for (int l = 0; l < D; ++l) {
            // level l occupies heap positions [2^l, 2^(l+1)): word 0 up to level 4, then
            // word 1, words 2-3, words 4-7
            uint32_t wsel;
            if (l < 5 || NW == 1) wsel = word[0];
            else if (l == 5) wsel = word[1 % NW];
            else if (l == 6) wsel = (h & 32u) ? word[3 % NW] : word[2 % NW];
            else {
                const uint32_t lo = (h & 32u) ? word[5 % NW] : word[4 % NW];
                const uint32_t hi = (h & 32u) ? word[7 % NW] : word[6 % NW];
                wsel = (h & 64u) ? hi : lo;
            }
            h = h + h + ((wsel >> (h & 31u)) & 1u);
        }
        const int leaf = (t << D) + static_cast<int>(h - N_POS);
        const TreeMeta tm = m.tree[t];
        if (LEAVES) {
            if (valid) leaf_out[row * T + tm.caller_tree] = m.leaf_node[leaf];
        } else {
            accu.add(m, tm.column, leaf);
        }
    }
    if (LEAVES) return;
    accu.flush();
    __syncthreads();
    if (wave == 0) finish_rows(m, lds.acc, row, valid, scores, labels, lane);
}

// ---------------------------------------------------------------------------------------
// Generic trees: any shape.  Outcome words are written to LDS (one word per 32 internal
// nodes, level order), the walk follows child references.
// ---------------------------------------------------------------------------------------
template <bool LEAVES, bool STAGED>
__global__ __launch_bounds__(BLOCK) void forest_generic_kernel(DevModel m, const float *__restrict__ X,
                                                               int64_t n_rows, float *scores,
                                                               int32_t *labels, int32_t *leaf_out)
{
    extern __shared__ __align__(16) char smem[];
    const Lds lds = carve_lds(smem, m, STAGED, true);
    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * TILE;
    const int64_t row = row0 + lane;
    const bool valid = row < n_rows;
    const int F = m.n_features;

    if (STAGED) {
        stage_x_tile(lds.xs, X, row0, n_rows, F);
        __syncthreads();
    }
    const float *xrow = X + (valid ? row : row0) * F;

    Accumulator accu;
    accu.init(lds.acc, wave, lane, m);
    uint32_t *mybits = lds.bits + static_cast<size_t>(wave) * m.max_words * TILE;

    const int T = m.n_trees;
    const int t_begin = static_cast<int>((static_cast<int64_t>(T) * wave) / WAVES);
    const int t_end = static_cast<int>((static_cast<int64_t>(T) * (wave + 1)) / WAVES);

    for (int t = t_begin; t < t_end; ++t) {
        const TreeMeta tm = m.tree[t];
        const SplitEntry *__restrict__ p = m.prog + tm.prog_base;
        for (int w = 0; w < tm.n_words; ++w) {
            uint32_t b = 0;
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                const SplitEntry e = p[w * 32 + j];
                const float x = STAGED ? lds.xs[e.feature_slot + lane] : xrow[e.feature_slot >> 6];
                b = b + b + (!(x <= e.threshold) ? 1u : 0u);
            }
            mybits[w * TILE + lane] = b;
        }
        // walk over child references; a validated tree ends within FOREST_MAX_DEPTH steps
        int ref = tm.root_ref;
        const ChildRef *__restrict__ ch = m.child + tm.child_base;
        for (int step = 0; step <= FOREST_MAX_DEPTH; ++step) {
            const bool inside = ref >= 0;
            if (!__any(inside)) break;
            if (inside) {
                const uint32_t wv = mybits[(ref >> 5) * TILE + lane];
                const ChildRef c = ch[ref];
                ref = ((wv >> (ref & 31)) & 1u) ? c.right : c.left;
            }
        }
        const int leaf = tm.leaf_base + (ref < 0 ? ~ref : 0);
        if (LEAVES) {
            if (valid) leaf_out[row * T + tm.caller_tree] = m.leaf_node[leaf];
        } else {
            accu.add(m, tm.column, leaf);
        }
    }
    if (LEAVES) return;
    accu.flush();
    __syncthreads();
    if (wave == 0) finish_rows(m, lds.acc, row, valid, scores, labels, lane);
}

constexpr size_t LDS_LIMIT = 160 * 1024;  // LDS of one gfx950 compute unit
size_t g_lds_limit = LDS_LIMIT;            // replaced by the device's per-workgroup limit at init

size_t lds_bytes(int kind, int n_features, int n_outputs, int max_words, bool staged)
{
    size_t b = sizeof(double) * WAVES * n_outputs * TILE;
    if (staged) b += sizeof(float) * n_features * TILE;
    if (kind == KIND_GENERIC) b += sizeof(uint32_t) * WAVES * max_words * TILE;
    return b;
}

size_t lds_bytes(const DevModel &m, bool staged)
{
    return lds_bytes(m.kind, m.n_features, m.n_outputs, m.max_words, staged);
}

using KernelFn = void (*)(DevModel, const float *, int64_t, float *, int32_t *, int32_t *);

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

bool model_fits(const PackedModel &m)
{
    return lds_bytes(m.kind, m.n_features, m.n_outputs, m.max_words, false) <= LDS_LIMIT;
}

hipError_t init_kernels()
{
    int dev = 0, per_block = 0;
    hipError_t e0 = hipGetDevice(&dev);
    if (e0 != hipSuccess) return e0;
    e0 = hipDeviceGetAttribute(&per_block, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e0 != hipSuccess) return e0;
    g_lds_limit = static_cast<size_t>(per_block) < LDS_LIMIT ? static_cast<size_t>(per_block) : LDS_LIMIT;
    for (int kind = 0; kind <= FULL_MAX_DEPTH; ++kind)
        for (int leaves = 0; leaves < 2; ++leaves)
            for (int staged = 0; staged < 2; ++staged) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick(kind, leaves, staged)),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   static_cast<int>(g_lds_limit));
                if (e != hipSuccess) return e;
            }
    return hipSuccess;
}

hipError_t launch_predict(const DevModel &m, const float *X, int64_t n_rows, float *scores,
                          int32_t *labels, int32_t *leaf_out, hipStream_t stream)
{
    if (n_rows <= 0) return hipSuccess;
    bool staged = true;
    if (lds_bytes(m, true) > g_lds_limit) staged = false;
    const size_t lds = lds_bytes(m, staged);
    if (lds > g_lds_limit) return hipErrorInvalidValue;
    const int64_t n_blocks = (n_rows + TILE - 1) / TILE;
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    KernelFn fn = pick(m.kind, leaf_out != nullptr, staged);
    hipLaunchKernelGGL(fn, dim3(static_cast<unsigned>(n_blocks)), dim3(BLOCK), lds, stream, m, X, n_rows,
                       scores, labels, leaf_out);
    return hipGetLastError();
}

}  // namespace forest_impl
