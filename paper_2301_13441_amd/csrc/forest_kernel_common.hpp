// Device helpers shared by the kernel families: X tile staging, per-wave partial sums,
// cross-wave reduction + transform + store.
//
// A workgroup is 4 wavefronts.  It owns ROWS = 64 * R consecutive rows (lane l of every wave
// stands for rows l, l + 64, ... of the tile) and splits the trees over its waves; each wave
// keeps fp64 partial sums per output column, the partials meet in LDS.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"

namespace forest_impl {

constexpr int TILE = 64;   // lanes per wavefront
constexpr int WAVES = 4;   // wavefronts per workgroup
constexpr int BLOCK = TILE * WAVES;

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Copies rows [row0, row0 + rows) of row-major X into xs[f * rows + r] (coalesced global
// reads, transposed LDS writes); rows past n_rows read as 0.
__device__ __forceinline__ void stage_x_tile(float *xs, const float *X, int64_t row0, int64_t n_rows,
                                             int F, int rows)
{
    const int64_t left = n_rows - row0;
    const int rows_here = left < rows ? static_cast<int>(left) : rows;
    const int n_valid = rows_here * F;
    const float *src = X + row0 * F;
    for (int e = threadIdx.x; e < rows * F; e += BLOCK) {
        const int r = e / F, f = e - r * F;
        xs[f * rows + r] = (e < n_valid) ? src[e] : 0.0f;
    }
}

// The trees of wave `wave` (of n_waves) in this workgroup: the trees are dealt, in contiguous
// runs, over (split, wave) pairs; blockIdx.y is the split (0 when the launch is not split).
__device__ __forceinline__ void tree_range(const DevModel &m, int wave, int n_waves, int &t_begin, int &t_end)
{
    const int64_t T = m.n_trees;
    const int64_t unit = static_cast<int64_t>(blockIdx.y) * n_waves + wave;
    const int64_t units = static_cast<int64_t>(m.n_splits) * n_waves;
    t_begin = static_cast<int>((T * unit) / units);
    t_end = static_cast<int>((T * (unit + 1)) / units);
}

// Aggregate, label, transform, store for one row whose K summed leaf values are raw[k * stride];
// raw[] is overwritten with the aggregated values.
__device__ __forceinline__ void finish_values(const DevModel &m, double *raw, int64_t stride, int64_t row,
                                              float *scores, int32_t *labels)
{
    const int K = m.n_outputs;
    double best = 0.0;
    int best_k = 0;
    for (int k = 0; k < K; ++k) {
        double s = raw[k * stride];
        // a column no tree feeds: the mean over no trees adds nothing to the base score
        if (m.aggregate == FOREST_AGG_MEAN && m.col_trees[k] > 0.0) s = s / m.col_trees[k];
        s = static_cast<double>(m.base[k]) + s;
        raw[k * stride] = s;
        if (k == 0 || s > best) {
            best = s;
            best_k = k;
        }
    }
    if (labels) {
        int lab = best_k;
        if (K == 1) lab = (m.transform == FOREST_TRANSFORM_SIGMOID) ? (best > 0.0) : (best > 0.5);
        labels[row] = lab;
    }
    if (!scores) return;
    float *dst = scores + row * K;
    if (m.transform == FOREST_TRANSFORM_SOFTMAX) {
        double z = 0.0;
        for (int k = 0; k < K; ++k) z += exp(raw[k * stride] - best);
        for (int k = 0; k < K; ++k) dst[k] = static_cast<float>(exp(raw[k * stride] - best) / z);
    } else if (m.transform == FOREST_TRANSFORM_SIGMOID) {
        for (int k = 0; k < K; ++k) dst[k] = static_cast<float>(1.0 / (1.0 + exp(-raw[k * stride])));
    } else {
        for (int k = 0; k < K; ++k) dst[k] = static_cast<float>(raw[k * stride]);
    }
}

// Tile row `li` (0 <= li < rows) once its K column sums are in acc[k * rows + li]: the rest of
// the row (aggregate, label, transform, store) or, in a split launch, the store of the sums.
__device__ __forceinline__ void finish_summed_row(const DevModel &m, double *acc, int rows, int li, int64_t row,
                                                  bool valid, float *scores, int32_t *labels)
{
    const int K = m.n_outputs;
    if (!valid) return;
    if (m.n_splits > 1) {
        double *dst = m.partial + (static_cast<int64_t>(blockIdx.y) * m.split_rows + row) * K;
        for (int k = 0; k < K; ++k) dst[k] = acc[k * rows + li];
        return;
    }
    finish_values(m, acc + li, rows, row, scores, labels);
}

// Cross-wave reduction for tile row `li`, then finish_summed_row.  `acc` is [n_waves][K][rows];
// wave 0's slice is overwritten.
__device__ __forceinline__ void finish_row(const DevModel &m, double *acc, int rows, int li, int64_t row,
                                           bool valid, float *scores, int32_t *labels, int n_waves = WAVES)
{
    const int K = m.n_outputs;
    for (int k = 0; k < K; ++k) {
        double s = acc[(0 * K + k) * rows + li];
        for (int w = 1; w < n_waves; ++w) s += acc[(w * K + k) * rows + li];
        acc[k * rows + li] = s;
    }
    finish_summed_row(m, acc, rows, li, row, valid, scores, labels);
}

// Partial sums of one wave for R rows per lane.  Scalar leaves accumulate in a register per
// run of trees that feed the same column (trees are sorted by column); vector leaves go
// straight to the wave's LDS slice.
template <int R>
struct Accumulator {
    double run[R];
    int col = 0;
    double *mine;  // this wave's [K][rows] slice
    int lane, K, W;
    static constexpr int rows = TILE * R;

    __device__ __forceinline__ void init(double *acc, int wave, int lane_, const DevModel &m)
    {
        K = m.n_outputs;
        W = m.leaf_width;
        lane = lane_;
        mine = acc + static_cast<size_t>(wave) * K * rows;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            run[r] = 0.0;
            for (int k = 0; k < K; ++k) mine[k * rows + r * TILE + lane] = 0.0;
        }
    }
    // `column` is wave-uniform; call once per tree before add()
    __device__ __forceinline__ void begin_tree(int column)
    {
        if (W == 1 && column != col) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                mine[col * rows + r * TILE + lane] += run[r];
                run[r] = 0.0;
            }
            col = column;
        }
    }
    // adds the payload of leaf `leaf` (index into the per-leaf tables) for row slot r
    __device__ __forceinline__ void add(const DevModel &m, int r, int leaf)
    {
        if (W == 1) {
            run[r] += static_cast<double>(m.leaf_value[leaf]);
        } else {
            const float *v = m.leaf_value + static_cast<size_t>(leaf) * K;
            for (int k = 0; k < K; ++k) mine[k * rows + r * TILE + lane] += static_cast<double>(v[k]);
        }
    }
    // scalar leaves only: adds a leaf value that was fetched earlier
    __device__ __forceinline__ void add_value(int r, float v) { run[r] += static_cast<double>(v); }
    __device__ __forceinline__ void flush()
    {
        if (W == 1) {
#pragma unroll
            for (int r = 0; r < R; ++r) mine[col * rows + r * TILE + lane] += run[r];
        }
    }
};

// The heap walk of a full tree of depth D over outcome words laid out by heap position:
// level l occupies positions [2^l, 2^(l+1)), i.e. word 0 up to level 4, then word 1,
// words 2-3, words 4-7.  Returns the heap position reached, 2^D + in-order leaf ordinal.
template <int D, int NW>
__device__ __forceinline__ uint32_t heap_walk_pos(const uint32_t (&word)[NW])
{
    uint32_t h = 1;
#pragma unroll
    for (int l = 0; l < D; ++l) {
        uint32_t wsel;
        if (l < 5 || NW == 1) wsel = word[0];
        else if (l == 5) wsel = word[1 % NW];
        else if (l == 6) wsel = (h & 32u) ? word[3 % NW] : word[2 % NW];
        else {
            const uint32_t lo = (h & 32u) ? word[5 % NW] : word[4 % NW];
            const uint32_t hi = (h & 32u) ? word[7 % NW] : word[6 % NW];
            wsel = (h & 64u) ? hi : lo;
        }
        h = h + h + __builtin_amdgcn_ubfe(wsel, h, 1u);  // bit (h mod 32) of the word
    }
    return h;
}

// The same walk, returning the in-order leaf ordinal.
template <int D, int NW>
__device__ __forceinline__ uint32_t heap_walk(const uint32_t (&word)[NW])
{
    return heap_walk_pos<D, NW>(word) - (1u << D);
}

using KernelFn = void (*)(DevModel, const float *, int64_t, float *, int32_t *, int32_t *);

}  // namespace forest_impl
