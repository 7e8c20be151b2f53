// Kernels that only split launches (small batches) use: threshold ranks per row tile, and the
// sum of the tree shares' partial sums.
//
// A batch of a few thousand rows has too few 128-row tiles to fill 256 compute units, so the
// trees are cut into shares as well (grid y of the family kernels).  Two things are then done
// once per batch instead of once per workgroup: the threshold ranks of the rank families are
// computed here, one thread per (row, feature), and left in global memory for every share's
// workgroup to load; and the shares' fp64 partial sums are added up here and the rows finished.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"
#include "forest_kernel_common.hpp"
#include "forest_rank_common.hpp"

namespace forest_impl {
namespace {

constexpr int RT_FEATURES = 2;           // features per workgroup: 256 threads = 128 rows x 2
constexpr int RT_MAX_PIVOTS = RANK_MAX_PIVOTS;

// grid (row tiles, ceil(F / 2)).  Same two-level search as rank_rows: the pivots of the
// workgroup's features staged in LDS, then one block of the sorted table in global memory.
__global__ __launch_bounds__(256) void forest_rank_tiles_kernel(DevModel m, const float *__restrict__ X,
                                                                int64_t n_rows)
{
    __shared__ float piv[RT_MAX_PIVOTS];
    const int F = m.n_features;
    const int f_first = blockIdx.y * RT_FEATURES;
    const int f_last = f_first + RT_FEATURES < F ? f_first + RT_FEATURES : F;
    const int piv_first = m.feat_pivot_base[f_first];
    const int piv_count = m.feat_pivot_base[f_last] - piv_first;
    for (int i = threadIdx.x; i < piv_count; i += 256) piv[i] = m.pivots[piv_first + i];
    __syncthreads();

    const int r = threadIdx.x & (RROWS - 1);  // row of the tile
    const int f = f_first + (threadIdx.x >> 7);
    if (f >= F) return;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * RROWS + r;
    const float x = row < n_rows ? X[row * F + f] : 0.0f;
    const int tb = m.feat_thr_base[f];
    const int n_thr = m.feat_thr_base[f + 1] - tb;
    const int pb = m.feat_pivot_base[f] - piv_first;
    int lo = 0, hi = m.feat_pivot_base[f + 1] - m.feat_pivot_base[f];
    while (lo < hi) {  // first block whose last threshold is not below x
        const int mid = (lo + hi) >> 1;
        if (piv[pb + mid] < x) lo = mid + 1;
        else hi = mid;
    }
    const int block = 1 << m.pivot_shift;
    lo = lo << m.pivot_shift;
    hi = lo + block < n_thr ? lo + block : n_thr;
    if (lo > hi) lo = hi;  // x is above every pivot: rank = n_thr
    while (lo < hi) {      // position inside the block
        const int mid = (lo + hi) >> 1;
        if (m.thr_sorted[tb + mid] < x) lo = mid + 1;
        else hi = mid;
    }
    const int rank = (x != x) ? n_thr : lo;  // NaN is right of every threshold
    const int reg0 = m.feat_vfirst[f];
    uint16_t *tile16 = reinterpret_cast<uint16_t *>(m.rank_tiles + static_cast<size_t>(blockIdx.x) * m.rank_regs * TILE);
    for (int sgm = 0, first = 0; first < n_thr; ++sgm, first += RANK_SEG) {
        const int len = n_thr - first < RANK_SEG ? n_thr - first : RANK_SEG;
        int rv = rank - first;
        rv = rv < 0 ? 0 : (rv > len ? len : rv);
        // tile row r lives in lane r % 64, low half for r < 64, high half above
        tile16[((reg0 + sgm) * TILE + (r & (TILE - 1))) * 2 + (r >> 6)] = f16_bits(rv - RANK_BIAS);
    }
}

constexpr int RS_ROWS = 8;     // rows per workgroup of the reduction
constexpr int RS_LANES = 16;   // lanes that share one (row, column) sum

// 16 lanes per (row, column): lane g adds the shares g, g + 16, ... in ascending order, a
// butterfly adds the 16 partial results, then one thread per row finishes the row exactly as
// an unsplit launch does.  The order of the additions is fixed, so results are reproducible.
__global__ __launch_bounds__(256) void forest_reduce_splits_kernel(DevModel m, int64_t n_rows, float *scores,
                                                                   int32_t *labels)
{
    __shared__ double raw[RS_ROWS * FOREST_MAX_OUTPUTS];
    const int K = m.n_outputs;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RS_ROWS;
    const int g = threadIdx.x & (RS_LANES - 1);
    for (int pair = threadIdx.x / RS_LANES; pair < RS_ROWS * K; pair += 256 / RS_LANES) {
        const int rl = pair / K, k = pair - rl * K;
        const int64_t row = row0 + rl;
        double s = 0.0;
        if (row < n_rows)
            for (int sp = g; sp < m.n_splits; sp += RS_LANES) s += m.partial[(sp * m.split_rows + row) * K + k];
#pragma unroll
        for (int d = RS_LANES / 2; d >= 1; d >>= 1) s += __shfl_xor(s, d, RS_LANES);
        if (g == 0) raw[rl * K + k] = s;
    }
    __syncthreads();
    const int64_t row = row0 + threadIdx.x;
    if (threadIdx.x < RS_ROWS && row < n_rows) finish_values(m, raw + threadIdx.x * K, 1, row, scores, labels);
}

}  // namespace

hipError_t launch_rank_tiles(const DevModel &m, const float *X, int64_t n_rows, hipStream_t stream)
{
    if (m.rank_regs <= 0) return hipSuccess;  // no feature has a threshold
    if (m.n_pivots > RT_MAX_PIVOTS) return hipErrorInvalidValue;
    const int64_t n_tiles = (n_rows + RROWS - 1) / RROWS;
    const int f_groups = (m.n_features + RT_FEATURES - 1) / RT_FEATURES;
    hipLaunchKernelGGL(forest_rank_tiles_kernel, dim3(static_cast<unsigned>(n_tiles), static_cast<unsigned>(f_groups)),
                       dim3(256), 0, stream, m, X, n_rows);
    return hipGetLastError();
}

hipError_t launch_reduce_splits(const DevModel &m, int64_t n_rows, float *scores, int32_t *labels,
                                hipStream_t stream)
{
    const int64_t n_blocks = (n_rows + RS_ROWS - 1) / RS_ROWS;
    hipLaunchKernelGGL(forest_reduce_splits_kernel, dim3(static_cast<unsigned>(n_blocks)), dim3(256), 0, stream, m,
                       n_rows, scores, labels);
    return hipGetLastError();
}

}  // namespace forest_impl
