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

// grid (row tiles, features): 128 threads, one per row of the tile.
__global__ __launch_bounds__(RROWS) void forest_rank_tiles_kernel(DevModel m, const float *__restrict__ X,
                                                                  int64_t n_rows)
{
    const int F = m.n_features;
    const int f = blockIdx.y;
    const int r = threadIdx.x;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * RROWS + r;
    const float x = row < n_rows ? X[row * F + f] : 0.0f;
    uint16_t *tile16 = reinterpret_cast<uint16_t *>(m.rank_tiles + static_cast<size_t>(blockIdx.x) * m.rank_regs * TILE);
    store_rank(tile16, m, f, r, rank_of(m, f, x));
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
    const int64_t n_tiles = (n_rows + RROWS - 1) / RROWS;
    hipLaunchKernelGGL(forest_rank_tiles_kernel,
                       dim3(static_cast<unsigned>(n_tiles), static_cast<unsigned>(m.n_features)), dim3(RROWS), 0,
                       stream, m, X, n_rows);
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
