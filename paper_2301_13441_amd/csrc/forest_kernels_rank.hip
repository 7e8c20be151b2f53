// Rank kernels for full trees (gfx950): X rewritten, exactly, as per-feature threshold ranks.
//
// A comparison x <= tau only needs to know where x falls among the thresholds it can meet
// (Section 4.3.1, dtype rewriting, applied to the input): with the distinct thresholds of
// feature f sorted, rank(x) = #{i : tau_i < x}, and a node holding tau_j sends x right iff
// rank(x) > j.  Ranks and node indices are small integers, stored as f16 codes, and two rows
// share one register (low / high half), so one packed instruction handles two rows:
//     v_pk_fma_f16  d, rank[reg], 4.0, (-4 j', -4 j')  clamp   -- d = 1.0 iff rank > j  (step (2) of Fig. 2)
// (rank and j' as f16 codes, forest_model.hpp).
// The register is selected with the VGPR index mode (s_set_gpr_idx_on / _idx: M0 = wave-uniform
// register index), so step (1), the feature selection matmul(X, W1), costs no vector
// instruction.  The outcomes of 8 nodes are turned into 8 bits per row either by the matrix
// core (up to 64 rank registers: BitCollector, one MFMA per 8 nodes) or by a tree of packed
// fused multiply-adds (128 rank registers: RankStep, 1024 + bits in each half, first entry in
// bit 7).  Four such bytes make one 32-bit heap-ordered outcome word, the same words the other
// kernels use, and the walk, leaf gather and reduction are shared.
//
// Prologue: every workgroup computes the ranks of its 128 rows from per-feature bucket tables
// (forest_rank_common.hpp).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"
#include "forest_kernel_common.hpp"
#include "forest_rank_common.hpp"

namespace forest_impl {
namespace {

// Eight entries (one outcome byte) applied to the lane's two rows.
template <int NVR>
struct RankStep;

#define FOREST_RANK_ASM(B)                                                                       \
    "s_set_gpr_idx_on %[e0], 0x1\n\t" FOREST_RANK_CMP(B, 0) FOREST_RANK_IDX(1) FOREST_RANK_CMP(B, 1)    \
        FOREST_RANK_IDX(2) FOREST_RANK_CMP(B, 2) FOREST_RANK_IDX(3) FOREST_RANK_CMP(B, 3)              \
            FOREST_RANK_IDX(4) FOREST_RANK_CMP(B, 4) FOREST_RANK_IDX(5) FOREST_RANK_CMP(B, 5)          \
                FOREST_RANK_IDX(6) FOREST_RANK_CMP(B, 6) FOREST_RANK_IDX(7) FOREST_RANK_CMP(B, 7)      \
                    "s_set_gpr_idx_off\n\t"                                                      \
                    "v_pk_fma_f16 %[d0], %[d0], %[c2], %[d1]\n\t"                                \
                    "v_pk_fma_f16 %[d2], %[d2], %[c2], %[d3]\n\t"                                \
                    "v_pk_fma_f16 %[d4], %[d4], %[c2], %[d5]\n\t"                                \
                    "v_pk_fma_f16 %[d6], %[d6], %[c2], %[d7]\n\t"                                \
                    "v_pk_fma_f16 %[d0], %[d0], %[c4], %[d2]\n\t"                                \
                    "v_pk_fma_f16 %[d4], %[d4], %[c4], %[d6]\n\t"                                \
                    "v_pk_fma_f16 %[d0], %[d0], %[c16], %[d4]\n\t"                               \
                    "v_pk_add_f16 %[a], %[d0], %[c1024]"
#define FOREST_RANK_OUTS                                                                              \
    [a] "=v"(acc), [d0] "=&v"(d0), [d1] "=&v"(d1), [d2] "=&v"(d2), [d3] "=&v"(d3), [d4] "=&v"(d4), \
        [d5] "=&v"(d5), [d6] "=&v"(d6), [d7] "=&v"(d7)
#define FOREST_RANK_INS                                                                                   \
    [e0] "s"(q.e[0]), [e1] "s"(q.e[1]), [e2] "s"(q.e[2]), [e3] "s"(q.e[3]), [e4] "s"(q.e[4]),            \
        [e5] "s"(q.e[5]), [e6] "s"(q.e[6]), [e7] "s"(q.e[7]), [c2] "s"(0x40004000u), [c4] "s"(0x44004400u), \
        [c16] "s"(0x4c004c00u), [c1024] "s"(0x64006400u)

template <>
struct RankStep<2> {
    static __device__ __forceinline__ void step(uint32_t &acc, const Entry8 &q, const v32u (&x)[2])
    {
        uint32_t d0, d1, d2, d3, d4, d5, d6, d7;
        asm volatile(FOREST_RANK_ASM("v64")
                     : FOREST_RANK_OUTS
                     : FOREST_RANK_INS, "{v[64:95]}"(x[0]), "{v[96:127]}"(x[1]));
    }
};

template <>
struct RankStep<4> {
    static __device__ __forceinline__ void step(uint32_t &acc, const Entry8 &q, const v32u (&x)[4])
    {
        uint32_t d0, d1, d2, d3, d4, d5, d6, d7;
        // base v32: with 128 pinned registers the kernel must fit 168 VGPRs for 3 waves per SIMD
        asm volatile(FOREST_RANK_ASM("v32")
                     : FOREST_RANK_OUTS
                     : FOREST_RANK_INS, "{v[32:63]}"(x[0]), "{v[64:95]}"(x[1]), "{v[96:127]}"(x[2]),
                       "{v[128:159]}"(x[3]));
    }
};

enum { MODE_SCALAR = 0, MODE_VECTOR = 1, MODE_LEAVES = 2 };

// The wave's share of the trees: dense evaluation, walk, leaf gather.  One instantiation per
// output mode so that each loop only keeps the scalar registers it needs.
template <int D, int NVR, int MODE>
__device__ __forceinline__ void rank_trees(const DevModel &m, const v32u (&x)[NVR], Accumulator<2> &accu, int wave,
                                           int lane, int64_t row0, int64_t n_rows, int32_t *leaf_out)
{
    constexpr int R = 2;
    constexpr int N_ENT = (1 << D) < 8 ? 8 : (1 << D);  // entries per tree
    constexpr int NW = N_ENT < 32 ? 1 : N_ENT / 32;     // outcome words per tree and row
    constexpr int GW = N_ENT < 32 ? N_ENT / 8 : 4;      // 8-entry groups (outcome bytes) per word
    constexpr int NB = GW * 8;                          // entries per scalar load batch = one word
    const int T = m.n_trees;
    int t_begin, t_end;
    tree_range(m, wave, WAVES, t_begin, t_end);

    // The wave's trees are one contiguous stream of entries; the batch after the last one
    // read here is padding the host appended to the program.
    ProgPtr p = (ProgPtr)(m.prog32 + static_cast<size_t>(t_begin) * N_ENT);
    MetaPtr meta = (MetaPtr)m.tree;
    Batch<NB> cur = load_batch<NB>(p);
    // Scalar leaf values are fetched one tree ahead of their use, so the gather's latency is
    // covered by the next tree's comparisons.
    float pending[R];
#pragma unroll
    for (int r = 0; r < R; ++r) pending[r] = 0.0f;
    int pending_col = 0;
    for (int t = t_begin; t < t_end; ++t) {
        // scalar loads, in flight together with the first batch of the tree
        const int column = meta[t].column;
        const int caller_tree = meta[t].caller_tree;
        uint32_t word[R][NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            uint32_t g[GW];
            // first group, then issue the next word's loads, then the rest: the loads are in
            // flight while this word is evaluated
            RankStep<NVR>::step(g[0], cur.q[0], x);
            p += NB;
            const Batch<NB> nxt = load_batch<NB>(p);
#pragma unroll
            for (int gi = 1; gi < GW; ++gi) RankStep<NVR>::step(g[gi], cur.q[gi], x);
            cur = nxt;
            // low byte of each half = 8 outcome bits; gather the bytes of row A and of row B
            if (GW == 4) {
                const uint32_t t01 = __builtin_amdgcn_perm(g[1 % GW], g[0], 0x06020400u);  // A0 A1 B0 B1
                const uint32_t t23 = __builtin_amdgcn_perm(g[3 % GW], g[2 % GW], 0x06020400u);
                word[0][w] = __builtin_amdgcn_perm(t23, t01, 0x05040100u);
                word[1][w] = __builtin_amdgcn_perm(t23, t01, 0x07060302u);
            } else if (GW == 2) {
                const uint32_t t01 = __builtin_amdgcn_perm(g[1 % GW], g[0], 0x06020400u);
                word[0][w] = t01 & 0xffffu;
                word[1][w] = t01 >> 16;
            } else {
                word[0][w] = g[0] & 0xffu;
                word[1][w] = (g[0] >> 16) & 0xffu;
            }
        }
        if (MODE == MODE_SCALAR) {
            accu.begin_tree(pending_col);
#pragma unroll
            for (int r = 0; r < R; ++r) accu.add_value(r, pending[r]);
            pending_col = column;
        }
        // wave-uniform base of the tree's leaf values, shifted so that the heap position the
        // walk ends on indexes it directly: one vector instruction per gather address
        const float *lv = m.leaf_value + ((t << D) - (1 << D));
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t pos = heap_walk_pos<D, NW>(word[r]);
            if (MODE == MODE_SCALAR) {
                pending[r] = lv[pos];
                continue;
            }
            const int leaf = (t << D) + static_cast<int>(pos - (1u << D));
            if (MODE == MODE_LEAVES) {
                const int64_t row = row0 + r * TILE + lane;
                if (row < n_rows) leaf_out[row * T + caller_tree] = m.leaf_node[leaf];
            } else {
                accu.add(m, r, leaf);
            }
        }
    }
    if (MODE == MODE_SCALAR) {
        accu.begin_tree(pending_col);
#pragma unroll
        for (int r = 0; r < R; ++r) accu.add_value(r, pending[r]);
    }
}

// The same, with the outcome bits collected by the matrix core (32 or 64 rank registers: the
// wide kernel has no registers to spare for the weights).  A word's MFMAs are still running
// when its last comparison has issued, so the word is read, and walked, one group later:
// after the first comparisons of the next word, or of the next tree's first word, whose leaf
// gather in turn is consumed one tree after that.
template <int D, int NVR, int MODE>
__device__ __forceinline__ void rank_trees_mfma(const DevModel &m, const v32u (&x)[NVR], Accumulator<2> &accu, int wave,
                                                int lane, int64_t row0, int64_t n_rows, int32_t *leaf_out)
{
    constexpr int R = 2;
    constexpr int N_ENT = (1 << D) < 8 ? 8 : (1 << D);
    constexpr int NW = N_ENT < 32 ? 1 : N_ENT / 32;
    constexpr int GW = N_ENT < 32 ? N_ENT / 8 : 4;
    constexpr int NB = GW * 8;
    const int T = m.n_trees;
    int t_begin, t_end;
    tree_range(m, wave, WAVES, t_begin, t_end);
    if (t_begin >= t_end) return;

    BitCollector bits;
    bits.init(lane);
    ProgPtr p = (ProgPtr)(m.prog32 + static_cast<size_t>(t_begin) * N_ENT);
    MetaPtr meta = (MetaPtr)m.tree;
    Batch<NB> cur = load_batch<NB>(p);
    v4f lo = bits.bias, hi = bits.bias;
    uint32_t pos[R], sel[R];
    float pending[R];
#pragma unroll
    for (int r = 0; r < R; ++r) pos[r] = 1u, sel[r] = 0u, pending[r] = 0.0f;
    int pending_col = 0, prev_column = 0, prev_caller = 0;

    // reads the word the last four (or fewer) MFMAs produced and advances the walk by it
    auto finish_word = [&](int w) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            // below 32 outcomes the bits above them are never indexed by the walk
            const uint32_t word = GW == 4 ? __builtin_amdgcn_perm(__float_as_uint(hi[r]), __float_as_uint(lo[r]), 0x05040100u)
                                          : __float_as_uint(lo[r]);
            heap_walk_word<D>(w, word, pos[r], sel[r]);
        }
    };
    // the walk of tree tp has ended on pos[]: consume the leaf
    auto finish_tree = [&](int tp, int column, int caller_tree) {
        if (MODE == MODE_SCALAR) {
            accu.begin_tree(pending_col);
#pragma unroll
            for (int r = 0; r < R; ++r) accu.add_value(r, pending[r]);
            pending_col = column;
        }
        const float *lv = m.leaf_value + ((tp << D) - (1 << D));
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (MODE == MODE_SCALAR) {
                // wave-uniform base + 32-bit byte offset: the gather takes its base from scalar
                // registers and needs one vector instruction for the address (a tree's leaves
                // are within 1 KB of the base)
                const uint32_t off = pos[r] << 2;
                pending[r] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(lv) + off);
            } else {
                const int leaf = (tp << D) + static_cast<int>(pos[r] - (1u << D));
                if (MODE == MODE_LEAVES) {
                    const int64_t row = row0 + r * TILE + lane;
                    if (row < n_rows) leaf_out[row * T + caller_tree] = m.leaf_node[leaf];
                } else {
                    accu.add(m, r, leaf);
                }
            }
            pos[r] = 1u;
        }
    };

    for (int t = t_begin; t < t_end; ++t) {
        const int column = meta[t].column;
        const int caller_tree = meta[t].caller_tree;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            uint32_t d[8];
            rank_compare(d, cur.q[0], x);
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_sched_barrier(0);  // the reads of the previous word stay behind these comparisons
#endif
            if (w > 0) {
                finish_word(w - 1);
            } else if (t > t_begin) {
                finish_word(NW - 1);
                finish_tree(t - 1, prev_column, prev_caller);
            }
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_sched_barrier(0);
#endif
            lo = bits.template collect<0>(d, bits.bias);
            p += NB;
            const Batch<NB> nxt = load_batch<NB>(p);
            if (GW >= 2) {
                rank_compare(d, cur.q[1 % GW], x);
                lo = bits.template collect<1>(d, lo);
            }
            if (GW == 4) {
                rank_compare(d, cur.q[2 % GW], x);
                hi = bits.template collect<0>(d, bits.bias);
                rank_compare(d, cur.q[3 % GW], x);
                hi = bits.template collect<1>(d, hi);
            }
            cur = nxt;
        }
        prev_column = column;
        prev_caller = caller_tree;
    }
    finish_word(NW - 1);
    finish_tree(t_end - 1, prev_column, prev_caller);
    if (MODE == MODE_SCALAR) {
        accu.begin_tree(pending_col);
#pragma unroll
        for (int r = 0; r < R; ++r) accu.add_value(r, pending[r]);
    }
}

template <int D, int NVR, int MODE>
__device__ __forceinline__ void run_trees(const DevModel &m, const v32u (&x)[NVR], Accumulator<2> &accu, int wave,
                                          int lane, int64_t row0, int64_t n_rows, int32_t *leaf_out)
{
    if constexpr (NVR <= 2) rank_trees_mfma<D, NVR, MODE>(m, x, accu, wave, lane, row0, n_rows, leaf_out);
    else rank_trees<D, NVR, MODE>(m, x, accu, wave, lane, row0, n_rows, leaf_out);
}

// Register budget: 32, 64 or 128 pinned rank registers (NVR = 1, 2, 4) plus the working set must
// leave room for 5, 4 resp. 3 waves per SIMD (96, 128 resp. 168 VGPRs).
template <int D, int NVR>
__global__ __launch_bounds__(BLOCK, (NVR == 1 ? 5 : NVR == 2 ? 4 : 3)) void forest_rank_kernel(DevModel m, const float *__restrict__ X,
                                                            int64_t n_rows, float *scores,
                                                            int32_t *labels, int32_t *leaf_out)
{
    constexpr int R = 2;
    extern __shared__ __align__(16) char smem[];
    uint32_t *rk = reinterpret_cast<uint32_t *>(smem);  // [32 * NVR][64] packed ranks, then reused as:
    double *acc = reinterpret_cast<double *>(smem);     // [WAVES][K][128] partial sums

    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RROWS;

    if (m.n_splits > 1) {  // launch-uniform: the ranks of the tile are already in global memory
        load_rank_tile(rk, m, BLOCK);
    } else {
        // 128 rank registers: four features per wave and iteration, 16 per workgroup, so a line
        // of X is used up in two iterations and can be streamed past the L2
        rank_rows<WAVES, (NVR == 4 ? 4 : 2), NVR == 4>(rk, m, X, row0, n_rows, wave, lane);
    }
    __syncthreads();
    v32u x[NVR];
#pragma unroll
    for (int q = 0; q < NVR; ++q)
#pragma unroll
        for (int i = 0; i < 32; ++i) x[q][i] = rk[(q * 32 + i) * TILE + lane];
    __syncthreads();  // rk is dead from here on; acc takes its place

    Accumulator<R> accu;
    accu.init(acc, wave, lane, m);
    if (leaf_out != nullptr) {  // wave-uniform: debug output instead of scores
        run_trees<D, NVR, MODE_LEAVES>(m, x, accu, wave, lane, row0, n_rows, leaf_out);
        return;
    }
    if (m.leaf_width == 1) run_trees<D, NVR, MODE_SCALAR>(m, x, accu, wave, lane, row0, n_rows, nullptr);
    else run_trees<D, NVR, MODE_VECTOR>(m, x, accu, wave, lane, row0, n_rows, nullptr);
    accu.flush();
    __syncthreads();
    const int li = threadIdx.x;
    if (li < RROWS) finish_row(m, acc, RROWS, li, row0 + li, row0 + li < n_rows, scores, labels);
}

size_t rank_lds_bytes(const DevModel &m, int nvr)
{
    const size_t a = sizeof(double) * WAVES * m.n_outputs * RROWS;
    const size_t b = sizeof(uint32_t) * 32 * nvr * TILE;
    return a > b ? a : b;
}

template <int NVR>
KernelFn pick_depth(int d)
{
    switch (d) {
        case 1: return forest_rank_kernel<1, NVR>;
        case 2: return forest_rank_kernel<2, NVR>;
        case 3: return forest_rank_kernel<3, NVR>;
        case 4: return forest_rank_kernel<4, NVR>;
        case 5: return forest_rank_kernel<5, NVR>;
        case 6: return forest_rank_kernel<6, NVR>;
        case 7: return forest_rank_kernel<7, NVR>;
        case 8: return forest_rank_kernel<8, NVR>;
        default: return nullptr;
    }
}

KernelFn pick_rank(int nvr, int d) { return nvr == 1 ? pick_depth<1>(d) : nvr == 2 ? pick_depth<2>(d) : pick_depth<4>(d); }

int rank_nvr(const DevModel &m) { return m.rank_regs <= 32 ? 1 : m.rank_regs <= 64 ? 2 : 4; }

}  // namespace

hipError_t init_rank_kernels(size_t lds_limit)
{
    for (int nvr = 1; nvr <= 4; nvr *= 2)
        for (int d = 1; d <= FULL_MAX_DEPTH; ++d) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_rank(nvr, d)),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               static_cast<int>(lds_limit));
            if (e != hipSuccess) return e;
        }
    return hipSuccess;
}

hipError_t launch_rank(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                       int32_t *leaf_out, hipStream_t stream)
{
    if (m.rank_regs > RANK_MAX_REGS || m.kind < 1 || m.kind > FULL_MAX_DEPTH) return hipErrorInvalidValue;
    const int nvr = rank_nvr(m);
    KernelFn fn = pick_rank(nvr, m.kind);
    const int64_t n_blocks = (n_rows + RROWS - 1) / RROWS;
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(n_blocks), static_cast<unsigned>(m.n_splits));
    hipLaunchKernelGGL(fn, grid, dim3(BLOCK), rank_lds_bytes(m, nvr), stream, m, X, n_rows, scores, labels, leaf_out);
    return hipGetLastError();
}

}  // namespace forest_impl
