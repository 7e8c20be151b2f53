// Rank kernel for trees of any shape (gfx950): packed f16 threshold ranks held in LDS.
//
// Same exact rewrite of the comparison as forest_kernels_rank.hip (rank(x) > j instead of
// !(x <= tau_j), two rows per 32-bit word, v_pk_add_f16 with clamp as the comparison), for
// models whose rank tile does not fit the vector registers: up to 256 rank rows of 64 words
// sit in LDS and every entry of the split program reads its row
//     v_and_or_b32  a, entry, 0xff00, lane * 4          -- LDS address of the row, no scalar op
//     ds_read_b32   x, a
//     v_pk_add_f16  d, x, entry.hi  clamp               -- step (2) of Fig. 2 for two rows
//     v_pk_fma_f16  ...                                 -- 8 outcomes -> one outcome byte
// i.e. three vector instructions and one LDS read per (node, two rows).
//
// Trees are stored level by level (internal nodes in level order, Section 3.1.2; every level
// padded to whole groups of 8 entries).  After the last group of a level the wave has that
// level's outcome bytes in its LDS buffer and every lane moves from its node to the child the
// bits select (the bit-level form of picking the leaf with matmul(., W3) + argmax); a child
// reference is either the child's ordinal in the next level or a leaf.  One pass over the
// stream therefore resolves the leaf with a working set of one level.
//
// A workgroup is RANKLDS_WAVES wavefronts on 128 rows; the trees are split over the waves.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"
#include "forest_kernel_common.hpp"
#include "forest_rank_common.hpp"

namespace forest_impl {
namespace {

constexpr int LWAVES = RANKLDS_WAVES;
constexpr int LBLOCK = TILE * LWAVES;

#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) TreeMeta *MetaPtr;
#else
typedef const TreeMeta *MetaPtr;  // host pass: the kernel body is only parsed
#endif

struct Entry8 {
    uint32_t e[8];
};

// LDS between the rank tile and the partial sums: the pivots during the prologue, then one
// chunk of outcome bytes (8 groups x 2 rows x 64 lanes) per wave.
__host__ __device__ inline size_t ranklds_region2_bytes(int n_pivots)
{
    const size_t piv = sizeof(float) * static_cast<size_t>(n_pivots);
    const size_t buf = static_cast<size_t>(LWAVES) * 8 * 2 * 64;
    return ((piv > buf ? piv : buf) + 15) / 16 * 16;
}

// Every lane loads the same eight words (one 32-byte piece of the stream).
__device__ __forceinline__ Entry8 load_group(const uint32_t *__restrict__ p)
{
    const uint4 lo = *reinterpret_cast<const uint4 *>(p);
    const uint4 hi = *reinterpret_cast<const uint4 *>(p + 4);
    Entry8 q;
    q.e[0] = lo.x; q.e[1] = lo.y; q.e[2] = lo.z; q.e[3] = lo.w;
    q.e[4] = hi.x; q.e[5] = hi.y; q.e[6] = hi.z; q.e[7] = hi.w;
    return q;
}

// One entry of a pair of groups: address of its rank row into a scratch register, the read, and
// the comparison, which overwrites the entry with its outcome.
#define FOREST_LDS_ADDR(t, e) "v_and_or_b32 " t ", %[" e "], %[mask], %[l4]\n\t"
#define FOREST_LDS_READ(t) "ds_read_b32 " t ", " t "\n\t"
#define FOREST_LDS_CMP(t, e) "v_pk_add_f16 %[" e "], " t ", %[" e "] op_sel:[0,1] op_sel_hi:[1,1] clamp\n\t"

// Two groups of 8 entries for the lane's two rows: every entry is replaced by its comparison
// outcome (1.0 or 0.0 in each f16 half), which the matrix core then turns into one outcome byte
// per group and row (first entry in bit 7).  All 16 LDS reads are issued before the first
// comparison, so the LDS latency is paid once per pair; they land in v112..v127, which the
// statement names as clobbered.  LDS operations complete in order, whatever scalar loads are
// also outstanding: "at most 8 outstanding" means the first eight reads have returned.
//
// The entries arrive through the vector memory path (every lane loads the same words), not
// through scalar loads: vector loads are counted in vmcnt, so waiting for the LDS reads
// (lgkmcnt) never waits for the program stream, which is fetched one pair ahead.
__device__ __forceinline__ void eval_pair(Entry8 &q, Entry8 &r, uint32_t mask, uint32_t l4)
{
    asm volatile(
        FOREST_LDS_ADDR("v112", "e0") FOREST_LDS_ADDR("v113", "e1") FOREST_LDS_ADDR("v114", "e2")
        FOREST_LDS_ADDR("v115", "e3") FOREST_LDS_ADDR("v116", "e4") FOREST_LDS_ADDR("v117", "e5")
        FOREST_LDS_ADDR("v118", "e6") FOREST_LDS_ADDR("v119", "e7")
        FOREST_LDS_READ("v112") FOREST_LDS_READ("v113") FOREST_LDS_READ("v114") FOREST_LDS_READ("v115")
        FOREST_LDS_READ("v116") FOREST_LDS_READ("v117") FOREST_LDS_READ("v118") FOREST_LDS_READ("v119")
        FOREST_LDS_ADDR("v120", "f0") FOREST_LDS_ADDR("v121", "f1") FOREST_LDS_ADDR("v122", "f2")
        FOREST_LDS_ADDR("v123", "f3") FOREST_LDS_ADDR("v124", "f4") FOREST_LDS_ADDR("v125", "f5")
        FOREST_LDS_ADDR("v126", "f6") FOREST_LDS_ADDR("v127", "f7")
        FOREST_LDS_READ("v120") FOREST_LDS_READ("v121") FOREST_LDS_READ("v122") FOREST_LDS_READ("v123")
        FOREST_LDS_READ("v124") FOREST_LDS_READ("v125") FOREST_LDS_READ("v126") FOREST_LDS_READ("v127")
        "s_waitcnt lgkmcnt(8)\n\t"
        FOREST_LDS_CMP("v112", "e0") FOREST_LDS_CMP("v113", "e1") FOREST_LDS_CMP("v114", "e2")
        FOREST_LDS_CMP("v115", "e3") FOREST_LDS_CMP("v116", "e4") FOREST_LDS_CMP("v117", "e5")
        FOREST_LDS_CMP("v118", "e6") FOREST_LDS_CMP("v119", "e7")
        "s_waitcnt lgkmcnt(0)\n\t"
        FOREST_LDS_CMP("v120", "f0") FOREST_LDS_CMP("v121", "f1") FOREST_LDS_CMP("v122", "f2")
        FOREST_LDS_CMP("v123", "f3") FOREST_LDS_CMP("v124", "f4") FOREST_LDS_CMP("v125", "f5")
        FOREST_LDS_CMP("v126", "f6") FOREST_LDS_CMP("v127", "f7")
        : [e0] "+v"(q.e[0]), [e1] "+v"(q.e[1]), [e2] "+v"(q.e[2]), [e3] "+v"(q.e[3]), [e4] "+v"(q.e[4]),
          [e5] "+v"(q.e[5]), [e6] "+v"(q.e[6]), [e7] "+v"(q.e[7]), [f0] "+v"(r.e[0]), [f1] "+v"(r.e[1]),
          [f2] "+v"(r.e[2]), [f3] "+v"(r.e[3]), [f4] "+v"(r.e[4]), [f5] "+v"(r.e[5]), [f6] "+v"(r.e[6]),
          [f7] "+v"(r.e[7])
        : [mask] "v"(mask), [l4] "v"(l4)
        : "memory", "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122",
          "v123", "v124", "v125", "v126", "v127");
}

// Output modes.  SCALAR1 (one output column, scalar leaves) and VECTOR2 (vector leaves, at most
// two columns) keep their partial sums in registers until every wave is done, so the partial
// sums can reuse the LDS of the rank tile; GENERAL keeps them in an LDS region of its own.
enum { MODE_SCALAR1 = 0, MODE_VECTOR2 = 1, MODE_GENERAL = 2, MODE_LEAVES = 3 };

constexpr int CHUNK_GROUPS = 8;  // a level is walked in chunks of 8 groups = 64 nodes

template <int MODE>
__device__ __forceinline__ void ranklds_trees(const DevModel &m, uint8_t *bytes, Accumulator<2> &accu,
                                              double (&sum)[2][2], int wave, int lane, int64_t row0,
                                              int64_t n_rows, int32_t *leaf_out)
{
    const int T = m.n_trees;
    int t_begin, t_end;
    tree_range(m, wave, LWAVES, t_begin, t_end);
    if (t_begin >= t_end) return;
    MetaPtr meta = (MetaPtr)m.tree;
    const uint32_t mask = 0xff00u;
    const uint32_t l4 = static_cast<uint32_t>(lane) * 4u;

    // The wave's trees are one contiguous stream of groups; the group after the last one read
    // here is padding the host appended to the program.
    int pos = meta[t_begin].prog_base;  // stream position of the current group
    // number of groups of the wave's trees (n_words = number of groups of a tree); the last one
    // carries the closing flag of the last tree
    const int n_groups = (meta[t_end - 1].prog_base + meta[t_end - 1].n_words * 8 - pos) / 8;
    // Three pairs of groups in rotation: while one pair is evaluated the fetches of the next two
    // are in flight; a pair's registers are refilled as soon as the pair has been evaluated.
    const uint32_t *__restrict__ p = m.prog32 + pos;
    Entry8 pa0 = load_group(p), pa1 = load_group(p + 8);
    Entry8 pb0 = load_group(p + 16), pb1 = load_group(p + 24);
    Entry8 pc0 = load_group(p + 32), pc1 = load_group(p + 40);
    int t = t_begin;
    int level_start = pos;  // stream position of the current level's first entry
    int chunk = 0;          // chunk index inside the level
    int gi = 0;             // group index inside the chunk
    // ref: ordinal of the lane's node inside the current level; ~leaf once a leaf is reached;
    // WAITING once the lane has picked its child in this level.  The child references are
    // fetched when the chunk that holds the node is complete and consumed one group into the
    // next level (or at the end of the tree), so the gather's latency is covered.
    constexpr int WAITING = static_cast<int>(0x80000000u);
    int ref[2];
    ChildRef pair[2];
    uint32_t went_right[2];
    bool resolve = false;  // wave-uniform: a level has ended since the last resolution
    ref[0] = ref[1] = meta[t].root_ref;
    pair[0] = pair[1] = ChildRef{0, 0};
    went_right[0] = went_right[1] = 0;
    // what the walk does with a group once its outcome bytes are known
    auto consume = [&](v4f g, uint32_t flags) {
        // low mantissa byte = outcome byte, of row A in g[0] and of row B in g[1]
        bytes[(gi * 2 + 0) * TILE + lane] = static_cast<uint8_t>(__float_as_uint(g[0]));
        bytes[(gi * 2 + 1) * TILE + lane] = static_cast<uint8_t>(__float_as_uint(g[1]));
        ++gi;
        pos += 8;
        if (gi == CHUNK_GROUPS || (flags & 1u)) {  // chunk complete: lanes whose node is in it pick a child
            if (resolve) {
#pragma unroll
                for (int r = 0; r < 2; ++r)
                    if (ref[r] == WAITING) ref[r] = went_right[r] ? pair[r].right : pair[r].left;
                resolve = false;
            }
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                if (ref[r] >= 0 && (ref[r] >> 6) == chunk) {
                    const uint32_t b = bytes[(((ref[r] >> 3) & 7) * 2 + r) * TILE + lane];
                    pair[r] = m.child[level_start + ref[r]];
                    went_right[r] = (b >> (ref[r] & 7)) & 1u;
                    ref[r] = WAITING;
                }
            }
            ++chunk;
            gi = 0;
        }
        if (flags & 1u) {  // level complete: every lane that was on a node has picked its child
            resolve = true;
            level_start = pos;
            chunk = 0;
        }
        if (flags & 2u) {  // tree complete: every lane stands on a leaf
#pragma unroll
            for (int r = 0; r < 2; ++r)
                if (ref[r] == WAITING) ref[r] = went_right[r] ? pair[r].right : pair[r].left;
            resolve = false;
            const TreeMeta tm = meta[t];
            if (MODE == MODE_GENERAL) accu.begin_tree(tm.column);
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const int leaf = tm.leaf_base + (ref[r] < 0 ? ~ref[r] : 0);
                if (MODE == MODE_LEAVES) {
                    const int64_t row = row0 + r * TILE + lane;
                    if (row < n_rows) leaf_out[row * T + tm.caller_tree] = m.leaf_node[leaf];
                } else if (MODE == MODE_SCALAR1) {
                    sum[r][0] += static_cast<double>(m.leaf_value[leaf]);
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
        }
    };
    // The matrix core is still collecting a pair's bits when its comparisons have issued, so
    // the walk consumes every pair one pair late: after the comparisons of the next one.
    BitCollector bits;
    bits.init(lane);
    v4f prev_g0 = bits.bias, prev_g1 = bits.bias;
    uint32_t prev_f0 = 0, prev_f1 = 0;
    int prev_count = 0;  // wave-uniform: groups of the previous pair that belong to the wave
    auto one_pair = [&](Entry8 q, Entry8 r, int count) {
        const uint32_t f0 = static_cast<uint32_t>(uniform(static_cast<int>(q.e[0])));
        const uint32_t f1 = static_cast<uint32_t>(uniform(static_cast<int>(r.e[0])));
        eval_pair(q, r, mask, l4);
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_sched_barrier(0);
#endif
        if (prev_count > 0) consume(prev_g0, prev_f0);
        if (prev_count > 1) consume(prev_g1, prev_f1);
        prev_g0 = bits.template collect<0>(q.e, bits.bias);
        prev_g1 = bits.template collect<0>(r.e, bits.bias);
        prev_f0 = f0;
        prev_f1 = f1;
        prev_count = count;
    };
    // The fetches are unconditional (past the end of the wave's stream they read the next
    // wave's groups or the padding at the end of the program), so that the same number of
    // fetches is issued between a buffer's fill and its use on every path.
    static_assert(PROGRAM_PAD_ENTRIES >= 88, "the last fetches reach 87 entries past a wave's stream");
    for (int group = 0; group < n_groups; group += 6) {
        one_pair(pa0, pa1, n_groups - group);
        pa0 = load_group(p + 48);
        pa1 = load_group(p + 56);
        if (group + 2 < n_groups) one_pair(pb0, pb1, n_groups - group - 2);
        pb0 = load_group(p + 64);
        pb1 = load_group(p + 72);
        if (group + 4 < n_groups) one_pair(pc0, pc1, n_groups - group - 4);
        pc0 = load_group(p + 80);
        pc1 = load_group(p + 88);
        p += 48;
    }
    if (prev_count > 0) consume(prev_g0, prev_f0);
    if (prev_count > 1) consume(prev_g1, prev_f1);
}

__global__ __launch_bounds__(LBLOCK) void forest_ranklds_kernel(DevModel m, const float *__restrict__ X,
                                                                int64_t n_rows, float *scores,
                                                                int32_t *labels, int32_t *leaf_out)
{
    extern __shared__ __align__(16) char smem[];
    const int regs = m.rank_regs > 0 ? m.rank_regs : 1;
    const int K = m.n_outputs;
    // LDS: [ rank tile | pivots, later one outcome-byte chunk per wave | partial sums (GENERAL) ].
    // The rank tile must start at LDS address 0: eval_group forms addresses as
    // (row offset | lane * 4).  SCALAR1 / VECTOR2 put their partial sums over the rank tile once
    // every wave has finished.
    uint32_t *rk = reinterpret_cast<uint32_t *>(smem);
    char *region2 = smem + sizeof(uint32_t) * TILE * regs;
    const bool deferred = (m.leaf_width == 1 && K == 1) || (m.leaf_width == K && K <= 2 && m.leaf_width != 1);
    const size_t r2_bytes = ranklds_region2_bytes(m.n_pivots);
    double *acc = deferred ? reinterpret_cast<double *>(smem) : reinterpret_cast<double *>(region2 + r2_bytes);

    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RROWS;

    if (m.rank_regs == 0) rk[threadIdx.x & (TILE - 1)] = 0;  // the padding entries read row 0
    if (m.n_splits > 1) {  // launch-uniform: the ranks of the tile are already in global memory
        load_rank_tile(rk, m, LBLOCK);
    } else {
        float *piv = reinterpret_cast<float *>(region2);
        for (int i = threadIdx.x; i < m.n_pivots; i += LBLOCK) piv[i] = m.pivots[i];
        __syncthreads();
        rank_rows<LWAVES>(rk, piv, m, X, row0, n_rows, wave, lane);
    }
    __syncthreads();  // ranks complete; the pivots are dead, their space becomes the byte chunks

    uint8_t *bytes = reinterpret_cast<uint8_t *>(region2) + static_cast<size_t>(wave) * CHUNK_GROUPS * 2 * TILE;
    Accumulator<2> accu;
    double sum[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
    if (leaf_out != nullptr) {  // wave-uniform: debug output instead of scores
        ranklds_trees<MODE_LEAVES>(m, bytes, accu, sum, wave, lane, row0, n_rows, leaf_out);
        return;
    }
    if (deferred) {
        if (m.leaf_width == 1) ranklds_trees<MODE_SCALAR1>(m, bytes, accu, sum, wave, lane, row0, n_rows, nullptr);
        else ranklds_trees<MODE_VECTOR2>(m, bytes, accu, sum, wave, lane, row0, n_rows, nullptr);
        __syncthreads();  // no wave reads the rank tile any more
        for (int r = 0; r < 2; ++r)
            for (int k = 0; k < K; ++k) acc[(wave * K + k) * RROWS + r * TILE + lane] = sum[r][k];
    } else {
        accu.init(acc, wave, lane, m);
        ranklds_trees<MODE_GENERAL>(m, bytes, accu, sum, wave, lane, row0, n_rows, nullptr);
        accu.flush();
    }
    __syncthreads();
    const int li = threadIdx.x;
    if (li < RROWS) finish_row(m, acc, RROWS, li, row0 + li, row0 + li < n_rows, scores, labels, LWAVES);
}

}  // namespace

size_t ranklds_lds_bytes(const DevModel &m)
{
    const size_t regs = m.rank_regs > 0 ? m.rank_regs : 1;
    const int K = m.n_outputs;
    const bool deferred = (m.leaf_width == 1 && K == 1) || (m.leaf_width == K && K <= 2 && m.leaf_width != 1);
    const size_t sums = sizeof(double) * LWAVES * K * RROWS;
    const size_t front = sizeof(uint32_t) * TILE * regs + ranklds_region2_bytes(m.n_pivots);
    return deferred ? (front > sums ? front : sums) : front + sums;
}

hipError_t init_ranklds_kernels(size_t lds_limit)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(forest_ranklds_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_limit));
}

hipError_t launch_ranklds(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                          int32_t *leaf_out, size_t lds_limit, hipStream_t stream)
{
    const size_t lds = ranklds_lds_bytes(m);
    if (lds > lds_limit || m.rank_regs > RANKLDS_MAX_REGS) return hipErrorInvalidValue;
    const int64_t n_blocks = (n_rows + RROWS - 1) / RROWS;
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(forest_ranklds_kernel, dim3(static_cast<unsigned>(n_blocks), static_cast<unsigned>(m.n_splits)), dim3(LBLOCK), lds, stream, m,
                       X, n_rows, scores, labels, leaf_out);
    return hipGetLastError();
}

}  // namespace forest_impl
