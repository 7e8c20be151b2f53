// Rank kernel for trees of any shape (gfx950): packed f16 threshold ranks held in LDS.
//
// Same exact rewrite of the comparison as forest_kernels_rank.hip (rank(x) > j instead of
// !(x <= tau_j), two rows per 32-bit word, v_pk_fma_f16 with clamp as the comparison), for
// models whose rank tile does not fit the vector registers: up to 256 rank rows of 64 words
// sit in LDS and every entry of the split program reads its row
//     s_and_b32           m0, entry, 0xff00             -- byte offset of the row (64 words each)
//     ds_read_addtid_b32  x                             -- LDS[m0 + lane * 4]
//     v_pk_fma_f16        x, x, 4.0, entry.hi  clamp    -- step (2) of Fig. 2 for two rows
// i.e. one vector instruction and one LDS read per (node, two rows); the matrix core then turns
// the 8 outcome registers of a group into one outcome byte per row (forest_rank_common.hpp).
// The address is formed on the scalar side because the vector ALU is what the kernel is short
// of (about 80 % busy); the write of M0 needs one wait state before the read that uses it.
//
// Trees are stored level by level (internal nodes in level order, Section 3.1.2; every level
// padded to whole groups of 8 entries).  After the last group of a level the wave has that
// level's outcome bytes in its LDS buffer and every lane moves from its node to the child the
// bits select (the bit-level form of picking the leaf with matmul(., W3) + argmax); a child
// reference is either the child's ordinal in the next level or a leaf.  One pass over the
// stream therefore resolves the leaf with a working set of one level.
//
// A workgroup is 12 or 8 wavefronts on 128 rows (the host compiler chooses: 12 where two
// workgroups fit a CU's LDS, which with 80 vector registers per lane gives 6 waves per SIMD);
// the trees are split over the waves.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"
#include "forest_kernel_common.hpp"
#include "forest_rank_common.hpp"

namespace forest_impl {
namespace {

typedef uint32_t v16u __attribute__((ext_vector_type(16)));

#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) uint32_t *StreamPtr;
#else
typedef const uint32_t *StreamPtr;  // host pass: the kernel body is only parsed
#endif

// LDS between the rank tile and the partial sums: one chunk of outcome bytes (8 groups x 2 rows
// x 64 lanes) per wave.
__host__ __device__ inline size_t ranklds_region2_bytes(int waves)
{
    return static_cast<size_t>(waves) * 8 * 2 * 64;
}

// A pair of groups (16 entries) is evaluated from 16 scalar registers: s[36:51] for even pairs,
// s[52:67] for odd pairs.  One entry: the byte offset of its rank row (bits 8..15 of the entry)
// goes to M0, the LDS read adds lane * 4 by itself, and the comparison leaves the outcome (1.0 or
// 0.0 in each f16 half) in the register the read filled.
#define FOREST_LDS_FETCH(t, e) "s_and_b32 m0, " e ", 0xff00\n\ts_nop 0\n\tds_read_addtid_b32 " t "\n\t"
#define FOREST_LDS_CMP(t, e) "v_pk_fma_f16 " t ", " t ", 4.0, " e " op_sel:[0,0,1] op_sel_hi:[1,0,1] clamp\n\t"
#if !defined(FOREST_RANKLDS_CONSERVATIVE)
// Streaming form: the statement ends by fetching, into the register set it has just used, the pair
// after the next one (NEXT); the fetch lands while the code between two statements runs.
#define FOREST_LDS_PAIR_HEAD(SET, CUR) ""
#define FOREST_LDS_PAIR_TAIL(SET, NEXT) "s_load_dwordx16 " SET ", %[p], " NEXT
#else
// Conservative form: the statement fetches its own 16 entries (CUR) and waits for them; nothing
// is in flight when it ends, and the register set is an ordinary scratch of the statement.
#define FOREST_LDS_PAIR_HEAD(SET, CUR) "s_load_dwordx16 " SET ", %[p], " CUR "\n\ts_waitcnt lgkmcnt(0)\n\t"
#define FOREST_LDS_PAIR_TAIL(SET, NEXT) ""
#endif
#define FOREST_LDS_PAIR(S0, S1, S2, S3, S4, S5, S6, S7, S8, S9, S10, S11, S12, S13, S14, S15, SET, CUR, NEXT)      \
    FOREST_LDS_PAIR_HEAD(SET, CUR)                                                                                 \
    "s_mov_b32 %[f0], " S0 "\n\t"                                                                                \
    "s_mov_b32 %[f1], " S8 "\n\t"                                                                                \
    FOREST_LDS_FETCH("v64", S0) FOREST_LDS_FETCH("v65", S1) FOREST_LDS_FETCH("v66", S2) FOREST_LDS_FETCH("v67", S3)  \
    FOREST_LDS_FETCH("v68", S4) FOREST_LDS_FETCH("v69", S5) FOREST_LDS_FETCH("v70", S6) FOREST_LDS_FETCH("v71", S7)  \
    FOREST_LDS_FETCH("v72", S8) FOREST_LDS_FETCH("v73", S9) FOREST_LDS_FETCH("v74", S10)                            \
    FOREST_LDS_FETCH("v75", S11) FOREST_LDS_FETCH("v76", S12) FOREST_LDS_FETCH("v77", S13)                          \
    FOREST_LDS_FETCH("v78", S14) FOREST_LDS_FETCH("v79", S15)                                                       \
    "s_waitcnt lgkmcnt(8)\n\t"                                                                                    \
    FOREST_LDS_CMP("v64", S0) FOREST_LDS_CMP("v65", S1) FOREST_LDS_CMP("v66", S2) FOREST_LDS_CMP("v67", S3)          \
    FOREST_LDS_CMP("v68", S4) FOREST_LDS_CMP("v69", S5) FOREST_LDS_CMP("v70", S6) FOREST_LDS_CMP("v71", S7)          \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                                    \
    FOREST_LDS_CMP("v72", S8) FOREST_LDS_CMP("v73", S9) FOREST_LDS_CMP("v74", S10) FOREST_LDS_CMP("v75", S11)        \
    FOREST_LDS_CMP("v76", S12) FOREST_LDS_CMP("v77", S13) FOREST_LDS_CMP("v78", S14) FOREST_LDS_CMP("v79", S15)      \
    FOREST_LDS_PAIR_TAIL(SET, NEXT)

// Two groups of 8 entries for the lane's two rows.  All 16 LDS reads are issued before the
// first comparison, so the LDS latency is paid once per pair.  LDS operations complete in
// order, whatever scalar loads are also outstanding, so "at most 8 outstanding" means the first
// eight reads have returned; the closing "none outstanding" also completes the scalar load the
// PREVIOUS pair issued, i.e. the entries of the NEXT pair.  The statement ends by fetching, into
// the scalar registers it has just used, the entries of the pair after the next one (two pairs
// = 128 bytes ahead); that load is in flight while the compiler's code between two statements
// runs, which never touches those registers: they are carried from statement to statement as
// one 16-register value pinned to s[36:51] resp. s[52:67].
//
// d0, d1: the outcomes of the two groups, the matrix core's B operands.  f0, f1: the first
// entry of each group (its low byte holds the group's flags).  M0 is written by every entry; it is a
// register the compiler reserves -- it keeps nothing of its own in M0 across an inline-assembly
// statement, sets it immediately before each use it generates, and rejects it on a clobber list as
// having no effect -- so the statements may write it freely.
//
// The streaming form is sound only if the compiler's own code between two statements leaves
// s[36:67] alone; the build checks that on the generated assembly before it links and otherwise
// builds the conservative form (FOREST_RANKLDS_CONSERVATIVE), which needs no such promise.
#if !defined(FOREST_RANKLDS_CONSERVATIVE)
#define FOREST_LDS_OUTS_EVEN(set) , "+{s[36:51]}"(set)
#define FOREST_LDS_OUTS_ODD(set) , "+{s[52:67]}"(set)
#define FOREST_LDS_CLOBBERS_EVEN "memory"
#define FOREST_LDS_CLOBBERS_ODD "memory"
#else
#define FOREST_LDS_OUTS_EVEN(set)
#define FOREST_LDS_OUTS_ODD(set)
#define FOREST_LDS_CLOBBERS_EVEN                                                                              \
    "memory", "s36", "s37", "s38", "s39", "s40", "s41", "s42", "s43", "s44", "s45", "s46", "s47", "s48", "s49", \
        "s50", "s51"
#define FOREST_LDS_CLOBBERS_ODD                                                                               \
    "memory", "s52", "s53", "s54", "s55", "s56", "s57", "s58", "s59", "s60", "s61", "s62", "s63", "s64", "s65", \
        "s66", "s67"
#endif
__device__ __forceinline__ void eval_pair_even(v8i &d0, v8i &d1, uint32_t &f0, uint32_t &f1, v16u &set,
                                               StreamPtr p)
{
    asm volatile(FOREST_LDS_PAIR("s36", "s37", "s38", "s39", "s40", "s41", "s42", "s43", "s44", "s45", "s46", "s47",
                                 "s48", "s49", "s50", "s51", "s[36:51]", "0x0", "0x80")
                 : "={v[64:71]}"(d0), "={v[72:79]}"(d1), [f0] "=&s"(f0), [f1] "=&s"(f1) FOREST_LDS_OUTS_EVEN(set)
                 : [p] "s"(p)
                 : FOREST_LDS_CLOBBERS_EVEN);
}

__device__ __forceinline__ void eval_pair_odd(v8i &d0, v8i &d1, uint32_t &f0, uint32_t &f1, v16u &set,
                                              StreamPtr p)
{
    asm volatile(FOREST_LDS_PAIR("s52", "s53", "s54", "s55", "s56", "s57", "s58", "s59", "s60", "s61", "s62", "s63",
                                 "s64", "s65", "s66", "s67", "s[52:67]", "0x40", "0xc0")
                 : "={v[64:71]}"(d0), "={v[72:79]}"(d1), [f0] "=&s"(f0), [f1] "=&s"(f1) FOREST_LDS_OUTS_ODD(set)
                 : [p] "s"(p)
                 : FOREST_LDS_CLOBBERS_ODD);
}

// The first two pairs of a wave's stream into the two register sets (streaming form only).
__device__ __forceinline__ void load_first_pairs(v16u &even, v16u &odd, StreamPtr p)
{
#if !defined(FOREST_RANKLDS_CONSERVATIVE)
    asm volatile("s_load_dwordx16 s[36:51], %[p], 0x0\n\t"
                 "s_load_dwordx16 s[52:67], %[p], 0x40\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "={s[36:51]}"(even), "={s[52:67]}"(odd)
                 : [p] "s"(p)
                 : "memory");
#endif
}

// The last statements' fetches are still in flight: let them land before the registers are reused
// (streaming form only).
__device__ __forceinline__ void finish_stream(v16u &even, v16u &odd)
{
#if !defined(FOREST_RANKLDS_CONSERVATIVE)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+{s[36:51]}"(even), "+{s[52:67]}"(odd) : : "memory");
#endif
}

// Output modes.  SCALAR1 (one output column, scalar leaves) and VECTOR2 (vector leaves, at most
// two columns) keep their partial sums in registers until every wave is done, so the partial
// sums can reuse the LDS of the rank tile; GENERAL (wider vector leaves) keeps a [K][rows] slice
// per wave in an LDS region of its own; SCALARK (scalar leaves, several columns) keeps one sum per
// (wave, column the wave's trees feed).
enum { MODE_SCALAR1 = 0, MODE_VECTOR2 = 1, MODE_GENERAL = 2, MODE_LEAVES = 3, MODE_SCALARK = 4 };

// SCALARK: the trees are sorted by output column, so the run of trees a wave evaluates feeds the
// consecutive columns first .. last, and the sum of a column is complete when the next column
// begins.  The wave keeps the running sums of its current column in registers and stores them,
// once, to its own slot of that column: mine[(column - first) * 128 + row in tile].
struct ColumnRuns {
    double run[2];
    double *mine;
    int first, current;

    __device__ __forceinline__ void start(double *slots, int first_column)
    {
        mine = slots;
        first = current = first_column;
        run[0] = run[1] = 0.0;
    }
    __device__ __forceinline__ void store(int lane) const
    {
        mine[(current - first) * RROWS + lane] = run[0];
        mine[(current - first) * RROWS + TILE + lane] = run[1];
    }
    // `column` is wave-uniform and never decreases
    __device__ __forceinline__ void begin_tree(int column, int lane)
    {
        if (column == current) return;
        store(lane);
        run[0] = run[1] = 0.0;
        for (++current; current < column; ++current) store(lane);  // columns no tree of the forest feeds
    }
};

constexpr int CHUNK_GROUPS = RANKLDS_CHUNK_GROUPS;  // a level is walked in chunks of 8 groups = 64 nodes

// The trees (processing order) of wave `wave` of the workgroup.
template <int LWAVES>
__device__ __forceinline__ void wave_trees(const DevModel &m, int wave, int &t_begin, int &t_end)
{
    if (m.n_splits == 1) {  // launch-uniform: runs of about equal program length, cut at load time
        t_begin = m.wave_tree[wave];
        t_end = m.wave_tree[wave + 1];
    } else {
        tree_range(m, wave, LWAVES, t_begin, t_end);
    }
}

template <int MODE, int LWAVES>
__device__ __forceinline__ void ranklds_trees(const DevModel &m, uint8_t *bytes, Accumulator<2> &accu,
                                              ColumnRuns &runs, double (&sum)[2][2], int wave, int lane,
                                              int64_t row0, int64_t n_rows, int32_t *leaf_out)
{
    const int T = m.n_trees;
    int t_begin, t_end;
    wave_trees<LWAVES>(m, wave, t_begin, t_end);
    if (t_begin >= t_end) return;
    MetaPtr meta = (MetaPtr)m.tree;

    // The wave's trees are one contiguous stream of groups; the group after the last one read
    // here is padding the host appended to the program.
    int pos = meta[t_begin].prog_base;  // stream position of the current group
    // number of groups of the wave's trees (n_words = number of groups of a tree); the last one
    // carries the closing flag of the last tree
    const int n_groups = (meta[t_end - 1].prog_base + meta[t_end - 1].n_words * 8 - pos) / 8;
    // The stream lives in scalar registers, two pairs of groups (2 x 16 entries) at a time.
    StreamPtr p = (StreamPtr)(m.prog32 + pos);
    v16u set_even, set_odd;
    load_first_pairs(set_even, set_odd, p);
    int t = t_begin;
    // The child references are addressed relative to the current tree: wave-uniform table base of
    // the tree + a per-lane 32-bit byte offset.  A tree's stream is its internal nodes plus at most
    // 7 entries of padding per level (at most 64 levels), far below the 2^29 entries the offset
    // can span, whatever the length of the whole program.
    const ChildRef *tree_child = m.child + pos;
    int level_start = 0;    // position of the current level's first entry inside the tree's stream
    int tree_start = pos;   // stream position of the tree's first entry
    int chunk = 0;          // chunk index inside the level
    int gi = 0;             // group index inside the chunk
    // ref: ordinal of the lane's node inside the current level; ~leaf once a leaf is reached;
    // WAITING once the lane has picked its child in this level.  The child references are
    // fetched when the chunk that holds the node is complete and consumed one group into the
    // next level (or at the end of the tree), so the gather's latency is covered.
    constexpr int WAITING = static_cast<int>(0x80000000u);
    int ref[2];
    ChildRef pair[2];
    uint32_t outcome[2], bit[2];  // the outcome byte that holds the lane's node, and the node's bit in it
    bool resolve = false;  // wave-uniform: a level has ended since the last resolution
    ref[0] = ref[1] = meta[t].root_ref;
    pair[0] = pair[1] = ChildRef{0, 0};
    outcome[0] = outcome[1] = bit[0] = bit[1] = 0;
    // what the walk does with a group once its outcome bytes are known
    auto consume = [&](v4f g, uint32_t flags) {
        // low mantissa byte = outcome byte, of row A in g[0] and of row B in g[1]
        bytes[(gi * 2 + 0) * TILE + lane] = static_cast<uint8_t>(__float_as_uint(g[0]));
        bytes[(gi * 2 + 1) * TILE + lane] = static_cast<uint8_t>(__float_as_uint(g[1]));
        ++gi;
        pos += 8;
        // flag bit 2: last group of a chunk (set at load time: every eighth group of a level and
        // its last).  Level and tree ends are chunk ends too, so the common group tests one bit.
        if (!(flags & 4u)) return;
        // chunk complete: lanes whose node is in it pick a child
        if (resolve) {
#pragma unroll
            for (int r = 0; r < 2; ++r)
                if (ref[r] == WAITING) ref[r] = ((outcome[r] >> bit[r]) & 1u) ? pair[r].right : pair[r].left;
            resolve = false;
        }
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            // the lane stands on node ref[r] of this chunk: 64 * chunk <= ref[r] < 64 * chunk + 64
            // (leaves and WAITING have the top bit set and fail the unsigned test)
            if ((static_cast<uint32_t>(ref[r]) ^ (static_cast<uint32_t>(chunk) << 6)) < 64u) {
                // both fetches are only looked at when the child is picked, a group or more later
                const uint32_t group_in_chunk = __builtin_amdgcn_ubfe(static_cast<uint32_t>(ref[r]), 3, 3);
                outcome[r] = bytes[group_in_chunk * (2 * TILE) + (r * TILE + lane)];
                bit[r] = static_cast<uint32_t>(ref[r]) & 7u;
                // wave-uniform base of the tree + 32-bit byte offset: one vector instruction for
                // the address instead of a 64-bit sum
                pair[r] = *reinterpret_cast<const ChildRef *>(
                    reinterpret_cast<const char *>(tree_child) + (static_cast<uint32_t>(level_start + ref[r]) << 3));
                ref[r] = WAITING;
            }
        }
        ++chunk;
        gi = 0;
        if (flags & 1u) {  // level complete: every lane that was on a node has picked its child
            resolve = true;
            level_start = pos - tree_start;
            chunk = 0;
        }
        if (flags & 2u) {  // tree complete: every lane stands on a leaf
#pragma unroll
            for (int r = 0; r < 2; ++r)
                if (ref[r] == WAITING) ref[r] = ((outcome[r] >> bit[r]) & 1u) ? pair[r].right : pair[r].left;
            resolve = false;
            const TreeMeta tm = meta[t];
            if (MODE == MODE_GENERAL) accu.begin_tree(tm.column);
            if (MODE == MODE_SCALARK) runs.begin_tree(tm.column, lane);
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int leaf = tm.leaf_base + (ref[r] < 0 ? ~ref[r] : 0);
                if (MODE == MODE_LEAVES) {
                    const int64_t row = row0 + r * TILE + lane;
                    if (row < n_rows) leaf_out[row * T + tm.caller_tree] = m.leaf_node[leaf];
                } else if (MODE == MODE_SCALAR1) {
                    sum[r][0] += static_cast<double>(m.leaf_value[leaf]);
                } else if (MODE == MODE_SCALARK) {
                    runs.run[r] += static_cast<double>(m.leaf_value[leaf]);
                } else if (MODE == MODE_VECTOR2) {
                    const float *v = m.leaf_value + static_cast<size_t>(leaf) * m.n_outputs;
                    sum[r][0] += static_cast<double>(v[0]);
                    if (m.n_outputs > 1) sum[r][1] += static_cast<double>(v[1]);
                } else {
                    accu.add(m, r, leaf);
                }
            }
            ++t;  // the metadata table has one spare record after the last tree
            ref[0] = ref[1] = meta[t].root_ref;
            tree_start = pos;
            tree_child = m.child + pos;
            level_start = 0;
        }
    };
    // The matrix core is still collecting a pair's bits when its comparisons have issued, so
    // the walk consumes every pair one pair late: after the comparisons of the next one.
    BitCollector bits;
    bits.init(lane);
    v4f prev_g0 = bits.bias, prev_g1 = bits.bias;
    uint32_t prev_f0 = 0, prev_f1 = 0;
    auto consume_previous = [&]() {
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_sched_barrier(0);
#endif
        consume(prev_g0, prev_f0);
        consume(prev_g1, prev_f1);
    };
    auto collect = [&](const v8i &d0, const v8i &d1, uint32_t f0, uint32_t f1) {
        prev_g0 = bits.collect_b(d0, bits.bias);
        prev_g1 = bits.collect_b(d1, bits.bias);
        prev_f0 = f0;
        prev_f1 = f1;
    };
    // Pair k of the wave's stream is evaluated from the even register set when k is even.  Every
    // statement fetches two pairs ahead whatever the wave's own group count is (past the end
    // of the wave's stream that is the next wave's groups or the padding at the end of the
    // program).  Every pair but the last has two groups of the wave's own.
    static_assert(PROGRAM_PAD_ENTRIES >= 64, "the last fetches reach 4 pairs past a wave's stream");
    const int n_pairs = (n_groups + 1) >> 1;
    v8i d0, d1;
    uint32_t f0, f1;
    eval_pair_even(d0, d1, f0, f1, set_even, p);
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_sched_barrier(0);
#endif
    collect(d0, d1, f0, f1);
    int k = 1;
    for (; k + 1 < n_pairs; k += 2) {
        eval_pair_odd(d0, d1, f0, f1, set_odd, p);
        consume_previous();
        collect(d0, d1, f0, f1);
        p += 32;
        eval_pair_even(d0, d1, f0, f1, set_even, p);
        consume_previous();
        collect(d0, d1, f0, f1);
    }
    if (k < n_pairs) {
        eval_pair_odd(d0, d1, f0, f1, set_odd, p);
        consume_previous();
        collect(d0, d1, f0, f1);
    }
    finish_stream(set_even, set_odd);
    consume(prev_g0, prev_f0);
    if (!(n_groups & 1)) consume(prev_g1, prev_f1);
}

// 80 vector registers per lane in either size: six waves per SIMD.
template <int LWAVES>
__global__ __launch_bounds__(TILE *LWAVES) __attribute__((amdgpu_waves_per_eu(6, 6))) void forest_ranklds_kernel(
    DevModel m, const float *__restrict__ X, int64_t n_rows, float *scores, int32_t *labels, int32_t *leaf_out)
{
    constexpr int LBLOCK = TILE * LWAVES;
    extern __shared__ __align__(16) char smem[];
    const int regs = m.rank_regs > 0 ? m.rank_regs : 1;
    const int K = m.n_outputs;
    // LDS: [ rank tile | one outcome-byte chunk per wave | partial sums (GENERAL, SCALARK) ].
    // The rank tile must start at LDS address 0: the entries' reads address it as
    // row offset + lane * 4.  SCALAR1 / VECTOR2 put their partial sums over the rank tile once
    // every wave has finished.
    uint32_t *rk = reinterpret_cast<uint32_t *>(smem);
    char *region2 = smem + sizeof(uint32_t) * TILE * regs;
    const bool deferred = (m.leaf_width == 1 && K == 1) || (m.leaf_width == K && K <= 2 && m.leaf_width != 1);
    const bool column_runs = m.leaf_width == 1 && K > 1;
    const size_t r2_bytes = ranklds_region2_bytes(LWAVES);
    double *acc = deferred ? reinterpret_cast<double *>(smem) : reinterpret_cast<double *>(region2 + r2_bytes);
    // SCALARK: (wave, column) sums [LWAVES + K - 1][128], summed columns [K][128], then per wave its
    // first column, its number of columns and its first slot
    double *slots = acc;
    double *summed = slots + static_cast<size_t>(LWAVES + K - 1) * RROWS;
    int *wave_first = reinterpret_cast<int *>(summed + static_cast<size_t>(K) * RROWS);
    int *wave_count = wave_first + LWAVES;
    int *wave_slot = wave_count + LWAVES;

    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RROWS;

    if (column_runs && leaf_out == nullptr && lane == 0) {  // which columns the wave's trees feed
        int t_begin, t_end;
        wave_trees<LWAVES>(m, wave, t_begin, t_end);
        const bool any = t_begin < t_end;
        wave_first[wave] = any ? m.tree[t_begin].column : 0;
        wave_count[wave] = any ? m.tree[t_end - 1].column - m.tree[t_begin].column + 1 : 0;
    }
    if (m.rank_regs == 0) rk[threadIdx.x & (TILE - 1)] = 0;  // the padding entries read row 0
    if (m.n_splits > 1) {  // launch-uniform: the ranks of the tile are already in global memory
        load_rank_tile(rk, m, LBLOCK);
    } else {
        // many features: four at a time per wave (8 lookups in flight per lane)
        rank_rows<LWAVES, 4>(rk, m, X, row0, n_rows, wave, lane);
    }
    __syncthreads();  // ranks complete

    uint8_t *bytes = reinterpret_cast<uint8_t *>(region2) + static_cast<size_t>(wave) * CHUNK_GROUPS * 2 * TILE;
    Accumulator<2> accu;
    ColumnRuns runs;
    double sum[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
    if (leaf_out != nullptr) {  // wave-uniform: debug output instead of scores
        ranklds_trees<MODE_LEAVES, LWAVES>(m, bytes, accu, runs, sum, wave, lane, row0, n_rows, leaf_out);
        return;
    }
    if (deferred) {
        if (m.leaf_width == 1)
            ranklds_trees<MODE_SCALAR1, LWAVES>(m, bytes, accu, runs, sum, wave, lane, row0, n_rows, nullptr);
        else
            ranklds_trees<MODE_VECTOR2, LWAVES>(m, bytes, accu, runs, sum, wave, lane, row0, n_rows, nullptr);
        __syncthreads();  // no wave reads the rank tile any more
        // constant indices into `sum` (K <= 2 here): indexed by a run-time k the array would
        // live in scratch memory and every tree would end with stores to it
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int k = 0; k < 2; ++k)
                if (k < K) acc[(wave * K + k) * RROWS + r * TILE + lane] = sum[r][k];
    } else if (column_runs) {
        int slot = 0;  // the slots of the waves before this one come first
        for (int v = 0; v < wave; ++v) slot += wave_count[v];
        if (lane == 0) wave_slot[wave] = slot;
        runs.start(slots + static_cast<size_t>(slot) * RROWS, wave_first[wave]);
        ranklds_trees<MODE_SCALARK, LWAVES>(m, bytes, accu, runs, sum, wave, lane, row0, n_rows, nullptr);
        if (wave_count[wave] > 0) runs.store(lane);  // the last column of the run
        __syncthreads();
        // column k of a row: the slots of the waves whose run covers k, in wave order
        const int li = threadIdx.x;
        if (li < RROWS) {
            for (int k = 0; k < K; ++k) {
                double s = 0.0;
                for (int v = 0; v < LWAVES; ++v) {
                    const int j = k - wave_first[v];
                    if (j >= 0 && j < wave_count[v]) s += slots[static_cast<size_t>(wave_slot[v] + j) * RROWS + li];
                }
                summed[k * RROWS + li] = s;
            }
            finish_summed_row(m, summed, RROWS, li, row0 + li, row0 + li < n_rows, scores, labels);
        }
        return;
    } else {
        accu.init(acc, wave, lane, m);
        ranklds_trees<MODE_GENERAL, LWAVES>(m, bytes, accu, runs, sum, wave, lane, row0, n_rows, nullptr);
        accu.flush();
    }
    __syncthreads();
    const int li = threadIdx.x;
    if (li < RROWS) finish_row(m, acc, RROWS, li, row0 + li, row0 + li < n_rows, scores, labels, LWAVES);
}

using RankLdsFn = void (*)(DevModel, const float *, int64_t, float *, int32_t *, int32_t *);

RankLdsFn ranklds_kernel_for(int waves)
{
    switch (waves) {
        case 12: return forest_ranklds_kernel<12>;
        case 8: return forest_ranklds_kernel<8>;
        case 4: return forest_ranklds_kernel<4>;
        case 2: return forest_ranklds_kernel<2>;
        default: return nullptr;
    }
}

}  // namespace

hipError_t init_ranklds_kernels(size_t lds_limit)
{
    for (int waves : RANKLDS_WAVE_CHOICES) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(ranklds_kernel_for(waves)),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_limit));
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_ranklds(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                          int32_t *leaf_out, size_t lds_limit, hipStream_t stream)
{
    RankLdsFn fn = ranklds_kernel_for(m.lds_waves);
    if (!fn) return hipErrorInvalidValue;
    const size_t lds = ranklds_lds_bytes(m.rank_regs, m.n_outputs, m.leaf_width, m.lds_waves);
    if (lds > lds_limit || m.rank_regs > RANKLDS_MAX_REGS) return hipErrorInvalidValue;
    const int64_t n_blocks = (n_rows + RROWS - 1) / RROWS;
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(n_blocks), static_cast<unsigned>(m.n_splits));
    hipLaunchKernelGGL(fn, grid, dim3(TILE * m.lds_waves), lds, stream, m, X, n_rows, scores, labels, leaf_out);
    return hipGetLastError();
}

}  // namespace forest_impl
