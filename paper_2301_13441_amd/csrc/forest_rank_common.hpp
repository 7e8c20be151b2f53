// Prologue shared by the rank kernel families: threshold ranks of a 128-row tile.
//
// rank(x) = #{i : tau_i < x} over the sorted distinct thresholds of a feature (all of them for
// NaN).  A node with threshold tau_j sends x right iff rank(x) > j, which is the float32
// comparison !(x <= tau_j) for every x; ranks are stored as exact f16 integers, two rows per
// 32-bit register (see forest_pack.cpp for the segment encoding).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"
#include "forest_kernel_common.hpp"

namespace forest_impl {

constexpr int RROWS = 128;  // rows per workgroup: lane l holds rows l (low half) and l + 64 (high half)

__device__ __forceinline__ uint16_t f16_bits(int v)
{
    const _Float16 h = static_cast<_Float16>(static_cast<float>(v));  // exact for |v| <= 2048
    return __builtin_bit_cast(uint16_t, h);
}

// Ranks of rows [row0, row0 + 128) for every feature with thresholds, written as f16 halves
// into rk[reg * 64 + (r & 63)] (low half: rows 0..63 of the tile, high half: rows 64..127).
// Two-level search: first over the feature's pivots (LDS: the last threshold of every block
// of 2^pivot_shift), then inside one block of the sorted table (global memory).
template <int THREADS>
__device__ __forceinline__ void rank_rows(uint32_t *rk, const float *piv, const DevModel &m,
                                          const float *__restrict__ X, int64_t row0, int64_t n_rows)
{
    constexpr int U = 8;  // searches in flight per thread
    const int F = m.n_features;
    const int64_t left = n_rows - row0;
    const int n_valid = (left < RROWS ? static_cast<int>(left) : RROWS) * F;
    const float *src = X + row0 * F;
    uint16_t *rk16 = reinterpret_cast<uint16_t *>(rk);
    const int block = 1 << m.pivot_shift;
    for (int e0 = threadIdx.x; e0 < RROWS * F; e0 += THREADS * U) {
        float x[U];
        int lo[U], hi[U], base[U], n_thr[U], f[U], r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * THREADS;
            const bool in = e < RROWS * F;
            r[u] = in ? e / F : 0;
            f[u] = in ? e - r[u] * F : 0;
            x[u] = (e < n_valid) ? src[e] : 0.0f;
            base[u] = m.feat_pivot_base[f[u]];
            lo[u] = 0;
            hi[u] = in ? m.feat_pivot_base[f[u] + 1] - base[u] : 0;
        }
        // first block whose last threshold is not below x
        for (int s = 0; s < m.rank_steps; ++s) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (lo[u] < hi[u]) {
                    const int mid = (lo[u] + hi[u]) >> 1;
                    if (piv[base[u] + mid] < x[u]) lo[u] = mid + 1;
                    else hi[u] = mid;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            base[u] = m.feat_thr_base[f[u]];
            n_thr[u] = (e0 + u * THREADS < RROWS * F) ? m.feat_thr_base[f[u] + 1] - base[u] : 0;
            lo[u] = lo[u] << m.pivot_shift;
            hi[u] = lo[u] + block < n_thr[u] ? lo[u] + block : n_thr[u];
            if (lo[u] > hi[u]) lo[u] = hi[u];  // x is above every pivot: rank = number of thresholds
        }
        // position inside the block
        for (int s = 0; s <= m.pivot_shift; ++s) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (lo[u] < hi[u]) {
                    const int mid = (lo[u] + hi[u]) >> 1;
                    if (m.thr_sorted[base[u] + mid] < x[u]) lo[u] = mid + 1;
                    else hi[u] = mid;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = e0 + u * THREADS;
            if (e >= RROWS * F) continue;
            const int rank = (x[u] != x[u]) ? n_thr[u] : lo[u];  // NaN is right of every threshold
            const int reg0 = m.feat_vfirst[f[u]];
            for (int s = 0, first = 0; first < n_thr[u]; ++s, first += RANK_SEG) {
                const int len = n_thr[u] - first < RANK_SEG ? n_thr[u] - first : RANK_SEG;
                int rv = rank - first;
                rv = rv < 0 ? 0 : (rv > len ? len : rv);
                rk16[((reg0 + s) * TILE + (r[u] & 63)) * 2 + (r[u] >> 6)] = f16_bits(rv - RANK_BIAS);
            }
        }
    }
}

}  // namespace forest_impl
