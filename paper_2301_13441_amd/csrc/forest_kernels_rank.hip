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

#ifndef FOREST_WIDE_FMA_TREE
#define FOREST_WIDE_FMA_TREE 0
#endif

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

// ---------------------------------------------------------------------------------------
// 128 rank registers (v32..v159): bit collection on the matrix core within 168 registers.
//
// Three waves per SIMD leave 40 registers beside the ranks, too few for two weight matrices, a
// four-register addend and compiler-placed accumulators.  So this kernel places its matrix-core
// operands by hand and uses ONE weight matrix: rows 4q and 4q + 1 of A weigh the row-a / row-b
// bytes of 16-lane block q by 2^(7 - v), rows 4q + 2 and 4q + 3 weigh them by 2^(15 - v), so a
// group's MFMA leaves its eight bits in the low byte of D[0], D[1] and in the second byte of D[2],
// D[3].  A chain of two groups is  D1 = A B1 + bias  into v[n:n+3], then  D2 = A B2 + C  with C =
// D = v[n+2:n+5]: the second group's low-byte sums land on the first group's second-byte sums, 16
// bits per row in v[n+2], v[n+3]; the other elements are never read.  Registers:
//     v[0:7]    the eight outcome registers of a group (B)
//     v[8:15]   A;  v[16:17] = 2^23, 2^23: the addend of a chain's first MFMA is v[14:17] (its
//               elements 0 and 1 only reach sums that are never read)
//     v[18:27]  accumulators: v[18:21] <- first group, v[20:23] <- second (bits in v20, v21),
//               v[22:25] <- third, v[24:27] <- fourth (bits in v24, v25)
// The compiler does not look inside a statement, so the waits the matrix core needs are written
// out: two idle states between a comparison and the MFMA that reads it, the 17 instructions of a
// group between an MFMA and the next one that reads or overwrites part of its result (12 states
// needed), and 12 idle states after a statement's last MFMA, since the compiler may read or copy
// the results right behind the statement.
// ---------------------------------------------------------------------------------------
typedef float v2f __attribute__((ext_vector_type(2)));
#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(1))) char *LeafBytes;  // global memory: loads with a scalar base
typedef const __attribute__((address_space(1))) float *LeafFloat;
#else
typedef const char *LeafBytes;  // host pass: the kernel body is only parsed
typedef const float *LeafFloat;
#endif

#define FOREST_WIDE_CMP(n, p) \
    "v_pk_fma_f16 v" #n ", v32, 4.0, %[" p #n "] op_sel:[0,0,1] op_sel_hi:[1,0,1] clamp\n\t"
#define FOREST_WIDE_IDX(n, p) "s_set_gpr_idx_idx %[" p #n "]\n\t"
#define FOREST_WIDE_GROUP(p)                                                                             \
    "s_set_gpr_idx_on %[" p "0], 0x1\n\t" FOREST_WIDE_CMP(0, p) FOREST_WIDE_IDX(1, p) FOREST_WIDE_CMP(1, p)   \
        FOREST_WIDE_IDX(2, p) FOREST_WIDE_CMP(2, p) FOREST_WIDE_IDX(3, p) FOREST_WIDE_CMP(3, p)               \
            FOREST_WIDE_IDX(4, p) FOREST_WIDE_CMP(4, p) FOREST_WIDE_IDX(5, p) FOREST_WIDE_CMP(5, p)           \
                FOREST_WIDE_IDX(6, p) FOREST_WIDE_CMP(6, p) FOREST_WIDE_IDX(7, p) FOREST_WIDE_CMP(7, p)       \
                    "s_set_gpr_idx_off\n\t"
#define FOREST_WIDE_MFMA(dst, c) \
    "s_nop 1\n\tv_mfma_f32_16x16x128_f8f6f4 " dst ", v[8:15], v[0:7], " c " cbsz:1 blgp:1\n\t"
#define FOREST_WIDE_ENTRIES(p, q)                                                                              \
    [p##0] "s"(q.e[0]), [p##1] "s"(q.e[1]), [p##2] "s"(q.e[2]), [p##3] "s"(q.e[3]), [p##4] "s"(q.e[4]),        \
        [p##5] "s"(q.e[5]), [p##6] "s"(q.e[6]), [p##7] "s"(q.e[7])
#define FOREST_WIDE_X "{v[32:63]}"(x[0]), "{v[64:95]}"(x[1]), "{v[96:127]}"(x[2]), "{v[128:159]}"(x[3])

struct WideCollector {
    v8i a;
    v2f bias;

    __device__ __forceinline__ void init(int lane)
    {
        const int m = lane & 15, q = lane >> 4;
        const bool mine = (m >> 2) == q;
        const int shift = (m & 1) == 0 ? 8 : 24;  // byte 1 = row a, byte 3 = row b
        const int up = (m & 2) ? 8 : 0;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const uint32_t bf8 = static_cast<uint32_t>(15 + up + 7 - v) << 2;  // 2^(up + 7 - v) in e5m2
            a[v] = mine ? static_cast<int>(bf8 << shift) : 0;
        }
        bias = v2f{8388608.0f, 8388608.0f};
        asm volatile("" : "+v"(bias));  // kept in registers instead of rebuilt before every statement
    }
    // The comparisons of the stream's very first group.
    __device__ __forceinline__ v8i first(const Entry8 &q, const v32u (&x)[4]) const
    {
        v8i d;
        asm volatile(FOREST_WIDE_GROUP("e") : "=&{v[0:7]}"(d) : FOREST_WIDE_ENTRIES(e, q), FOREST_WIDE_X);
        return d;
    }
    // One word of GW groups.  On entry d holds the outcomes of the word's first group (the one
    // that ends up in the higher byte of a chain); every MFMA is followed by the comparisons of the
    // next group, the last one by those of the NEXT word's first group, which d holds on return.
    // So the last MFMA is complete when the statement ends, and the wave has comparisons to issue
    // while it runs.  e.g[] are the groups in the order they are compared.  Returns the 16-bit
    // halves (GW = 4: lo and hi; GW = 2: lo) or, for GW = 1, the group's bits in the second byte of lo.
    template <int GW>
    __device__ __forceinline__ void word(v8i &d, const Entry8 (&g)[GW], const v32u (&x)[4], v2f &lo, v2f &hi) const
    {
        if constexpr (GW == 4) {
            asm volatile(FOREST_WIDE_MFMA("v[18:21]", "v[14:17]") FOREST_WIDE_GROUP("a")
                             FOREST_WIDE_MFMA("v[20:23]", "v[20:23]") FOREST_WIDE_GROUP("b")
                                 FOREST_WIDE_MFMA("v[22:25]", "v[14:17]") FOREST_WIDE_GROUP("c")
                                     FOREST_WIDE_MFMA("v[24:27]", "v[24:27]") FOREST_WIDE_GROUP("e")
                         : "={v[20:21]}"(lo), "={v[24:25]}"(hi), "+{v[0:7]}"(d)
                         : "{v[8:15]}"(a), "{v[16:17]}"(bias), FOREST_WIDE_ENTRIES(a, g[0]), FOREST_WIDE_ENTRIES(b, g[1 % GW]),
                           FOREST_WIDE_ENTRIES(c, g[2 % GW]), FOREST_WIDE_ENTRIES(e, g[3 % GW]), FOREST_WIDE_X
                         : "v18", "v19", "v22", "v23", "v26", "v27");
        } else if constexpr (GW == 2) {
            asm volatile(FOREST_WIDE_MFMA("v[18:21]", "v[14:17]") FOREST_WIDE_GROUP("a")
                             FOREST_WIDE_MFMA("v[20:23]", "v[20:23]") FOREST_WIDE_GROUP("b")
                         : "={v[20:21]}"(lo), "+{v[0:7]}"(d)
                         : "{v[8:15]}"(a), "{v[16:17]}"(bias), FOREST_WIDE_ENTRIES(a, g[0]), FOREST_WIDE_ENTRIES(b, g[1 % GW]),
                           FOREST_WIDE_X
                         : "v18", "v19", "v22", "v23");
        } else {
            asm volatile(FOREST_WIDE_MFMA("v[18:21]", "v[14:17]") FOREST_WIDE_GROUP("a")
                         : "={v[20:21]}"(lo), "+{v[0:7]}"(d)
                         : "{v[8:15]}"(a), "{v[16:17]}"(bias), FOREST_WIDE_ENTRIES(a, g[0]), FOREST_WIDE_X
                         : "v18", "v19");
        }
    }
};

// The groups one statement of WideCollector compares, for the word of GW groups at p: the word's
// groups after its first one in the order 0, 3, 2 (a chain takes its higher byte first), then
// group 1 of the next word (group 0 where a word is a single group).
template <int GW>
struct WideEntries {
    Entry8 g[GW];
};

__device__ __forceinline__ Entry8 load_group(ProgPtr p)
{
    Entry8 e;
#pragma unroll
    for (int j = 0; j < 8; ++j) e.e[j] = p[j];
    return e;
}

template <int GW>
__device__ __forceinline__ WideEntries<GW> load_wide(ProgPtr p)
{
    WideEntries<GW> e;
    if constexpr (GW == 4) {
        e.g[0] = load_group(p);
        e.g[1 % GW] = load_group(p + 24);
        e.g[2 % GW] = load_group(p + 16);
        e.g[3 % GW] = load_group(p + 32 + 8);
    } else if constexpr (GW == 2) {
        e.g[0] = load_group(p);
        e.g[1 % GW] = load_group(p + 16 + 8);
    } else {
        e.g[0] = load_group(p + 8);
    }
    return e;
}

// The wave's share of the trees with WideCollector.  A word's bits are complete when its
// statement ends, so the word is walked right away and a tree's leaf values are consumed one
// tree later.  The statement of the wave's last word compares one group of the next wave's trees
// or of the padding behind the program; nothing reads those outcomes.
template <int D, int MODE>
__device__ __forceinline__ void rank_trees_wide(const DevModel &m, const v32u (&x)[4], Accumulator<2> &accu, int wave,
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

    WideCollector bits;
    bits.init(lane);
    ProgPtr p = (ProgPtr)(m.prog32 + static_cast<size_t>(t_begin) * N_ENT);
    MetaPtr meta = (MetaPtr)m.tree;
    WideEntries<GW> cur = load_wide<GW>(p);
    v8i d = bits.first(load_group(p + (GW >= 2 ? 8 : 0)), x);
    float pending[R];
#pragma unroll
    for (int r = 0; r < R; ++r) pending[r] = 0.0f;
    int pending_col = 0;
    // wave-uniform base of the current tree's leaf values, shifted so that the heap position the
    // walk ends on indexes it directly; carried from tree to tree in scalar registers
    LeafBytes lv = (LeafBytes)(m.leaf_value + ((t_begin << D) - (1 << D)));

    for (int t = t_begin; t < t_end; ++t, lv += sizeof(float) << D) {
        asm volatile("" : "+s"(lv));
        const int column = meta[t].column;
        const int caller_tree = meta[t].caller_tree;
        uint32_t pos[R], sel[R];
#pragma unroll
        for (int r = 0; r < R; ++r) pos[r] = 1u, sel[r] = 0u;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            p += NB;
            const WideEntries<GW> nxt = load_wide<GW>(p);  // in flight during this word's statement
            v2f lo, hi;
            bits.template word<GW>(d, cur.g, x, lo, hi);
            cur = nxt;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                uint32_t word;
                if (GW == 4) word = __builtin_amdgcn_perm(__float_as_uint(hi[r]), __float_as_uint(lo[r]), 0x05040100u);
                else if (GW == 2) word = __float_as_uint(lo[r]);  // the bits above the 16 are never indexed
                else word = __float_as_uint(lo[r]) >> 8;
                heap_walk_word<D>(w, word, pos[r], sel[r]);
            }
            // a word is walked before the next one is evaluated: its halves are not copied aside
            if (D >= 7) asm volatile("" : "+v"(pos[0]), "+v"(pos[1]), "+v"(sel[0]), "+v"(sel[1]));
            else asm volatile("" : "+v"(pos[0]), "+v"(pos[1]));
        }
        if (MODE == MODE_SCALAR) {
            accu.begin_tree(pending_col);
#pragma unroll
            for (int r = 0; r < R; ++r) accu.add_value(r, pending[r]);
            pending_col = column;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (MODE == MODE_SCALAR) {
                const uint32_t off = pos[r] << 2;
                pending[r] = *(LeafFloat)(lv + off);
            } else {
                const int leaf = (t << D) + static_cast<int>(pos[r] - (1u << D));
                if (MODE == MODE_LEAVES) {
                    const int64_t row = row0 + r * TILE + lane;
                    if (row < n_rows) leaf_out[row * T + caller_tree] = m.leaf_node[leaf];
                } else {
                    accu.add(m, r, leaf);
                }
            }
        }
    }
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
    else if constexpr (FOREST_WIDE_FMA_TREE) rank_trees<D, NVR, MODE>(m, x, accu, wave, lane, row0, n_rows, leaf_out);
    else rank_trees_wide<D, MODE>(m, x, accu, wave, lane, row0, n_rows, leaf_out);
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
