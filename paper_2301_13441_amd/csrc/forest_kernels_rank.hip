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
// instruction.  The outcomes of 8 nodes are turned into 8 bits per row by the matrix core
// (HandCollector: one MFMA per 8 nodes, first entry in bit 7).  Four such bytes make one 32-bit
// outcome word.  Trees of depth 4..6 keep their bits in subtree fields and are walked three levels
// at a time through two small tables in LDS (the bit form of matmul(., W3) + argmax, Fig. 2 step
// (3)); depths 7 and 8 do so for their first five levels and go on with the bit walk of the other
// kernels, which depths 1..3 use throughout.  Leaf gather and reduction are shared.
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

enum { MODE_SCALAR = 0, MODE_VECTOR = 1, MODE_LEAVES = 2 };
constexpr int WALK_TABLE_BYTES = 512;  // 128 two-byte records and two tables of 128 bytes at the start of the LDS
// Depths 7, 8: every wave keeps the words behind a tree's first one in LDS, one dword per word and
// row ([word][row slot][lane], one spare word): which of them holds the field of a lane's level-5
// subtree differs from lane to lane, and registers cannot be indexed per lane.
constexpr int deep_words(int depth) { return depth > STAGED_MAX_DEPTH ? (1 << depth) / 32 : 0; }
constexpr int deep_bytes_per_wave(int depth) { return deep_words(depth) * 2 * TILE * 4; }

// ---------------------------------------------------------------------------------------
// Bit collection on the matrix core with operands placed by hand.
//
// The eight outcome registers of a group are, read as bytes, (0, a, 0, b) with a, b = 0x3c (1.0
// in bf8) or 0 for the lane's two rows.  v_mfma_f32_16x16x128_f8f6f4 takes them as its B operand:
// a lane of 16-lane block q supplies B[k][n] for n = lane % 16 and the 32 values of k that belong
// to block q, and receives D[4q + i][n], i = 0..3.  With an A that is zero outside A[4q + i][k of
// block q] every D only sums the lane's own bytes.  ONE weight matrix serves: rows 4q and 4q + 1
// weigh the row-a / row-b bytes by 2^(7 - v) (register v of the group: first entry in bit 7), rows
// 4q + 2 and 4q + 3 weigh them by 2^(15 - v), so a group's MFMA leaves its eight bits in the low
// byte of D[0], D[1] and in the second byte of D[2], D[3], on top of a 2^23 addend (exact: every
// partial sum is an integer below 2^24).  A chain of two groups is  D1 = A B1 + bias  into
// v[n:n+3], then  D2 = A B2 + C  with C = D = v[n+2:n+5]: the second group's low-byte sums land on
// the first group's second-byte sums, 16 bits per row in v[n+2], v[n+3]; the other elements are
// never read.  Registers (the rank registers follow from v28, v64 or, with 128 of them, v32 on,
// which leaves 40 for everything else at three waves per SIMD):
//     v[0:7]    the eight outcome registers of a group (B)
//     v[8:15]   A;  v[16:17] = 2^23, 2^23: the addend of a chain's first MFMA is v[14:17] (its
//               elements 0 and 1 only reach sums that are never read)
//     v[18:27]  accumulators: v[18:21] <- first group, v[20:23] <- second (bits in v20, v21),
//               v[22:25] <- third, v[24:27] <- fourth (bits in v24, v25)
// The compiler does not look inside a statement and knows of no matrix instruction here, so the
// waits the matrix core needs are in the statements: two idle states between a comparison and
// the MFMA that reads it, and the 18 instructions of a group between an MFMA and anything that
// reads or overwrites part of its result (12 states needed) -- every MFMA of a statement is
// followed by a group, the last one by the first group of the NEXT word, so its result is complete
// when the statement ends and the compiler may read or copy it at once.
// ---------------------------------------------------------------------------------------
typedef float v2f __attribute__((ext_vector_type(2)));
#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(1))) char *LeafBytes;  // global memory: loads with a scalar base
typedef const __attribute__((address_space(1))) float *LeafFloat;
#else
typedef const char *LeafBytes;  // host pass: the kernel body is only parsed
typedef const float *LeafFloat;
#endif

#define FOREST_HAND_CMP(B, n, p) \
    "v_pk_fma_f16 v" #n ", " B ", 4.0, %[" p #n "] op_sel:[0,0,1] op_sel_hi:[1,0,1] clamp\n\t"
#define FOREST_HAND_IDX(n, p) "s_set_gpr_idx_idx %[" p #n "]\n\t"
#define FOREST_HAND_GROUP(B, p)                                                                                   \
    "s_set_gpr_idx_on %[" p "0], 0x1\n\t" FOREST_HAND_CMP(B, 0, p) FOREST_HAND_IDX(1, p) FOREST_HAND_CMP(B, 1, p)      \
        FOREST_HAND_IDX(2, p) FOREST_HAND_CMP(B, 2, p) FOREST_HAND_IDX(3, p) FOREST_HAND_CMP(B, 3, p)                  \
            FOREST_HAND_IDX(4, p) FOREST_HAND_CMP(B, 4, p) FOREST_HAND_IDX(5, p) FOREST_HAND_CMP(B, 5, p)              \
                FOREST_HAND_IDX(6, p) FOREST_HAND_CMP(B, 6, p) FOREST_HAND_IDX(7, p) FOREST_HAND_CMP(B, 7, p)          \
                    "s_set_gpr_idx_off\n\t"
#define FOREST_HAND_MFMA(dst, c) \
    "s_nop 1\n\tv_mfma_f32_16x16x128_f8f6f4 " dst ", v[8:15], v[0:7], " c " cbsz:1 blgp:1\n\t"
#define FOREST_HAND_ENTRIES(p, q)                                                                              \
    [p##0] "s"(q.e[0]), [p##1] "s"(q.e[1]), [p##2] "s"(q.e[2]), [p##3] "s"(q.e[3]), [p##4] "s"(q.e[4]),        \
        [p##5] "s"(q.e[5]), [p##6] "s"(q.e[6]), [p##7] "s"(q.e[7])
#define FOREST_HAND_X1 "{v[28:59]}"(x[0])
#define FOREST_HAND_X2 "{v[64:95]}"(x[0]), "{v[96:127]}"(x[1 % NVR])
#define FOREST_HAND_X4 \
    "{v[32:63]}"(x[0]), "{v[64:95]}"(x[1 % NVR]), "{v[96:127]}"(x[2 % NVR]), "{v[128:159]}"(x[3 % NVR])

// The statements, for rank registers from B on, passed as the operands X.
#define FOREST_HAND_FIRST(B, X) \
    asm volatile(FOREST_HAND_GROUP(B, "e") : "=&{v[0:7]}"(d) : FOREST_HAND_ENTRIES(e, q), X)
#define FOREST_HAND_WORD4(B, X)                                                                                    \
    asm volatile(FOREST_HAND_MFMA("v[18:21]", "v[14:17]") FOREST_HAND_GROUP(B, "a")                                \
                     FOREST_HAND_MFMA("v[20:23]", "v[20:23]") FOREST_HAND_GROUP(B, "b")                            \
                         FOREST_HAND_MFMA("v[22:25]", "v[14:17]") FOREST_HAND_GROUP(B, "c")                        \
                             FOREST_HAND_MFMA("v[24:27]", "v[24:27]") FOREST_HAND_GROUP(B, "e")                    \
                 : "={v[20:21]}"(lo), "={v[24:25]}"(hi), "+{v[0:7]}"(d)                                          \
                 : "{v[8:15]}"(a), "{v[16:17]}"(bias), FOREST_HAND_ENTRIES(a, g[0]), FOREST_HAND_ENTRIES(b, g[1 % GW]), \
                   FOREST_HAND_ENTRIES(c, g[2 % GW]), FOREST_HAND_ENTRIES(e, g[3 % GW]), X                       \
                 : "v18", "v19", "v22", "v23", "v26", "v27")
#define FOREST_HAND_WORD2(B, X)                                                                                    \
    asm volatile(FOREST_HAND_MFMA("v[18:21]", "v[14:17]") FOREST_HAND_GROUP(B, "a")                                \
                     FOREST_HAND_MFMA("v[20:23]", "v[20:23]") FOREST_HAND_GROUP(B, "b")                            \
                 : "={v[20:21]}"(lo), "+{v[0:7]}"(d)                                                              \
                 : "{v[8:15]}"(a), "{v[16:17]}"(bias), FOREST_HAND_ENTRIES(a, g[0]), FOREST_HAND_ENTRIES(b, g[1 % GW]), X \
                 : "v18", "v19", "v22", "v23")
#define FOREST_HAND_WORD1(B, X)                                                                                    \
    asm volatile(FOREST_HAND_MFMA("v[18:21]", "v[14:17]") FOREST_HAND_GROUP(B, "a")                                \
                 : "={v[20:21]}"(lo), "+{v[0:7]}"(d)                                                              \
                 : "{v[8:15]}"(a), "{v[16:17]}"(bias), FOREST_HAND_ENTRIES(a, g[0]), X                            \
                 : "v18", "v19")

template <int NVR>
struct HandCollector {
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
    __device__ __forceinline__ v8i first(const Entry8 &q, const v32u (&x)[NVR]) const
    {
        v8i d;
        if constexpr (NVR == 4) FOREST_HAND_FIRST("v32", FOREST_HAND_X4);
        else if constexpr (NVR == 2) FOREST_HAND_FIRST("v64", FOREST_HAND_X2);
        else FOREST_HAND_FIRST("v28", FOREST_HAND_X1);
        return d;
    }
    // One word of GW groups.  On entry d holds the outcomes of the word's first group (the one
    // that ends up in the higher byte of a chain); every MFMA is followed by the comparisons of the
    // next group, the last one by those of the NEXT word's first group, which d holds on return.
    // g[] are the groups in the order they are compared.  Returns the 16-bit halves (GW = 4: lo
    // and hi; GW = 2: lo) or, for GW = 1, the group's bits in the second byte of lo.
    template <int GW>
    __device__ __forceinline__ void word(v8i &d, const Entry8 (&g)[GW], const v32u (&x)[NVR], v2f &lo, v2f &hi) const
    {
        if constexpr (GW == 4) {
            if constexpr (NVR == 4) FOREST_HAND_WORD4("v32", FOREST_HAND_X4);
            else if constexpr (NVR == 2) FOREST_HAND_WORD4("v64", FOREST_HAND_X2);
            else FOREST_HAND_WORD4("v28", FOREST_HAND_X1);
        } else if constexpr (GW == 2) {
            if constexpr (NVR == 4) FOREST_HAND_WORD2("v32", FOREST_HAND_X4);
            else if constexpr (NVR == 2) FOREST_HAND_WORD2("v64", FOREST_HAND_X2);
            else FOREST_HAND_WORD2("v28", FOREST_HAND_X1);
        } else {
            if constexpr (NVR == 4) FOREST_HAND_WORD1("v32", FOREST_HAND_X4);
            else if constexpr (NVR == 2) FOREST_HAND_WORD1("v64", FOREST_HAND_X2);
            else FOREST_HAND_WORD1("v28", FOREST_HAND_X1);
        }
    }
};

// The groups one statement of HandCollector compares, for the word of GW groups at p: the word's
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

// Makes the compiler place its wait for the loads of e here.
template <int GW>
__device__ __forceinline__ void wait_for(const WideEntries<GW> &e)
{
#pragma unroll
    for (int i = 0; i < GW; ++i)
        asm volatile("" : : "s"(e.g[i].e[0]), "s"(e.g[i].e[1]), "s"(e.g[i].e[2]), "s"(e.g[i].e[3]), "s"(e.g[i].e[4]),
                     "s"(e.g[i].e[5]), "s"(e.g[i].e[6]), "s"(e.g[i].e[7]));
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_sched_barrier(0);
#endif
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

// The wave's share of the trees.  A word's bits are complete when its statement ends, so the
// word is walked right away; a tree's leaf values are gathered at the end of its iteration and
// added one tree later.  The statement of the wave's last word compares one group of the next
// wave's trees or of the padding behind the program; nothing reads those outcomes.
//
// Scalar leaves: the trees are sorted by output column, so the wave's trees are a few runs of one
// column each (the runs' ends are the running sums of the columns' tree counts), and inside a
// run the loop over the trees is one basic block -- no test of the column per tree, and the
// requests for the next tree's entries stay in front of the statement they are to overlap.
template <int D, int NVR, int MODE>
__device__ __forceinline__ void rank_trees_hand(const DevModel &m, const v32u (&x)[NVR], Accumulator<2> &accu, int wave,
                                                int lane, int64_t row0, int64_t n_rows, int32_t *leaf_out,
                                                const uint8_t *walk_tables)
{
    constexpr bool STAGED = D >= STAGED_MIN_DEPTH && D <= STAGED_MAX_DEPTH;
    constexpr int R = 2;
    constexpr int N_ENT = (1 << D) < 8 ? 8 : (1 << D);
    constexpr int NW = N_ENT < 32 ? 1 : N_ENT / 32;
    constexpr int GW = N_ENT < 32 ? N_ENT / 8 : 4;
    constexpr int NB = GW * 8;
    const int T = m.n_trees;
    int t_begin, t_end;
    tree_range(m, wave, WAVES, t_begin, t_end);
    if (t_begin >= t_end) return;

    HandCollector<NVR> bits;
    bits.init(lane);
    ProgPtr p = (ProgPtr)(m.prog32 + static_cast<size_t>(t_begin) * N_ENT);
    WideEntries<GW> cur = load_wide<GW>(p);
    v8i d = bits.first(load_group(p + (GW >= 2 ? 8 : 0)), x);

    // The walk's tables, read at LDS addresses the instruction can hold: the tables are the first
    // thing in the kernel's LDS (address 0: the kernel has no static LDS, init_rank_kernels checks).
    // table(index, offset) is byte `offset + index` of them.
    auto table = [](uint32_t index, uint32_t offset) -> uint32_t {
#if defined(__HIP_DEVICE_COMPILE__)
        return *reinterpret_cast<const __attribute__((address_space(3))) uint8_t *>(static_cast<uintptr_t>(offset + index));
#else
        return index + offset;
#endif
    };
    (void)walk_tables;
    // the wave's strip for the words of deep trees, at a literal address plus the lane's: indexed
    // as an array, so that constant parts of an index end up in the instruction
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((address_space(3))) uint32_t *DeepPtr;
    typedef volatile __attribute__((address_space(3))) uint16_t *DeepHalfPtr;  // volatile: not merged back into words
#else
    typedef uint32_t *DeepPtr;  // host pass: the kernel body is only parsed
    typedef volatile uint16_t *DeepHalfPtr;
#endif
    const DeepPtr deep = (DeepPtr)(static_cast<uintptr_t>(WALK_TABLE_BYTES + wave * deep_bytes_per_wave(D) + lane * 4));
    // Whether the first table is read while the tree's second word is evaluated (two more registers
    // live across that statement; the 128-register kernel has none to spare and measured the same
    // either way).
    constexpr bool EARLY = NVR < 4 && NW == 2;

    // evaluates and walks the next tree of the stream: leaf4[r] = 4 x the ordinal of the leaf row r
    // ends on (depths 1..3: 4 x the heap position, 2^D + ordinal)
    auto walk_tree = [&](uint32_t (&leaf4)[R]) {
        uint32_t pos[R], word0[R], start[R], base4[R];
#pragma unroll
        for (int r = 0; r < R; ++r) pos[r] = 1u, word0[r] = 0u, start[r] = 0u, base4[r] = 0u;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            // Scalar loads return in any order, so the only wait there is waits for all of them: the
            // entries of this word are waited for (they were requested a statement ago) BEFORE the
            // next word's are requested, which then have the whole statement to arrive.
            wait_for(cur);
            if constexpr (STAGED && EARLY) {
                if (w == 1) {  // behind the wait, so that these reads are not waited for before the statement
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        const uint32_t top = word0[r] & 0xfeu;
                        start[r] = table(top, 0u);
                        base4[r] = table(top, 1u);
                    }
                }
            }
            p += NB;
            const WideEntries<GW> nxt = load_wide<GW>(p);
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_sched_barrier(0);  // requested before the statement, not behind it
#endif
            v2f lo, hi;
            bits.template word<GW>(d, cur.g, x, lo, hi);
            cur = nxt;
            uint32_t word[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if (D > STAGED_MAX_DEPTH && w > 0) word[r] = 0u;  // its halves go to LDS as they are
                else if (GW == 4) word[r] = __builtin_amdgcn_perm(__float_as_uint(hi[r]), __float_as_uint(lo[r]), 0x05040100u);
                else if (GW == 2) word[r] = __float_as_uint(lo[r]);  // the bits above the 16 are never indexed
                else word[r] = __float_as_uint(lo[r]) >> 8;
            }
            if constexpr (STAGED) {
                // Three levels at a time from two tables in LDS (forest_model.hpp has the bit
                // layout).  Bits 1..7 of the tree's first word are the outcomes of levels 0..2 and
                // index, times two, the table of two-byte records {where the field of the level-3
                // subtree they lead to begins, 4 x the ordinal of that subtree's first leaf}, read
                // byte by byte (an LDS read costs the vector ALU nothing, taking a 16-bit record
                // apart does); the field's bits index the table of 4 x the leaf's ordinal inside
                // the subtree.  Both tables span at most 64 banks once: lanes never collide.  The
                // reads of the two rows go out together.
                constexpr uint32_t FIELD = (1u << (D - 3)) - 1u;
                if (w == 0) {
#pragma unroll
                    for (int r = 0; r < R; ++r) word0[r] = word[r];
                }
                if (w == NW - 1) {
                    if (!EARLY) {
                        uint32_t top[R];
#pragma unroll
                        for (int r = 0; r < R; ++r) top[r] = word0[r] & 0xfeu;
#if defined(__HIP_DEVICE_COMPILE__)
                        __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            start[r] = table(top[r], 0u);
                            base4[r] = table(top[r], 1u);
                        }
#if defined(__HIP_DEVICE_COMPILE__)
                        __builtin_amdgcn_sched_barrier(0);
#endif
                    }
                    uint32_t inner[R], field[R];
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        // the shift and the extraction read the low 6 (5) bits of their count only
                        if (NW == 2)
                            field[r] = static_cast<uint32_t>(((static_cast<uint64_t>(word[r]) << 32) | word0[r]) >> (start[r] & 63u)) &
                                       ((1u << FIELD) - 1u);
                        else
                            field[r] = __builtin_amdgcn_ubfe(word[r], start[r], FIELD);
                    }
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);  // both rows' reads go out before either is waited for
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r) inner[r] = table(field[r], 256u);
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r) leaf4[r] = base4[r] + inner[r];
                    // one 32-bit sum per row, used as the offset of the gather (left to itself the
                    // compiler adds the two bytes to the 64-bit base one after the other)
                    asm volatile("" : "+v"(leaf4[0]), "+v"(leaf4[1]));
                }
            } else if constexpr (D > STAGED_MAX_DEPTH) {
                // Depths 7, 8.  The first word (levels 0..4) by the same two tables, which give the
                // ordinal of the level-5 subtree the row reaches.  The other words go to the wave's
                // strip of LDS as they come; after the last one every lane reads the two words its
                // subtree's field lies in (7 or 3 bits at 7 or 3 times the ordinal), and a third
                // table gives 4 x the leaf's ordinal inside the subtree.
                constexpr uint32_t DL = D - 5, DFIELD = (1u << DL) - 1u;
                if (w == 0) {
                    uint32_t top[R], field[R];
#pragma unroll
                    for (int r = 0; r < R; ++r) top[r] = word[r] & 0xfeu;
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        start[r] = table(top[r], 0u);
                        base4[r] = table(top[r], 1u);
                    }
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r) field[r] = __builtin_amdgcn_ubfe(word[r], start[r], 3u);  // reads 5 bits of start
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r) pos[r] = table(field[r], 256u);
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r) pos[r] += base4[r];  // ordinal of the level-5 subtree, 0..31
                } else {
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        // the word's two halves, stored as 16 bits each: no instruction to join them
                        const DeepHalfPtr half = (DeepHalfPtr)(deep + (w - 1) * (2 * TILE) + r * TILE);
                        half[0] = static_cast<uint16_t>(__float_as_uint(lo[r]));
                        half[1] = static_cast<uint16_t>(__float_as_uint(hi[r]));
                    }
                }
                if (w == NW - 1) {
                    uint32_t lo_w[R], hi_w[R], shift[R], field[R], inner[R];
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        uint32_t bit = pos[r] << DL;
                        asm volatile("" : "+v"(bit));  // (kept from being turned back into a 32-bit multiplication)
                        bit -= pos[r];                 // DFIELD x the ordinal: where the field begins
                        const DeepPtr at = deep + (bit >> 5) * (2 * TILE);
                        shift[r] = bit & 31u;
                        lo_w[r] = at[r * TILE];
                        hi_w[r] = at[r * TILE + 2 * TILE];                        // the spare word behind the last one
                    }
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r)
                        field[r] = static_cast<uint32_t>(((static_cast<uint64_t>(hi_w[r]) << 32) | lo_w[r]) >> shift[r]) &
                                   ((1u << DFIELD) - 1u);
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r) inner[r] = table(field[r], 384u);
#if defined(__HIP_DEVICE_COMPILE__)
                    __builtin_amdgcn_sched_barrier(0);
#endif
#pragma unroll
                    for (int r = 0; r < R; ++r) leaf4[r] = (pos[r] << (DL + 2)) + inner[r];
                    asm volatile("" : "+v"(leaf4[0]), "+v"(leaf4[1]));
                }
            } else {
                // Depths 1..3: one word in heap order (bit = heap index), one step per level.
#pragma unroll
                for (int r = 0; r < R; ++r) {
#pragma unroll
                    for (int l = 0; l < D; ++l) pos[r] = pos[r] + pos[r] + __builtin_amdgcn_ubfe(word[r], pos[r], 1u);
                    leaf4[r] = pos[r] << 2;
                }
            }
            // a word is dealt with before the next one is evaluated: its halves are not copied aside
            if constexpr (STAGED) asm volatile("" : "+v"(word0[0]), "+v"(word0[1]));
            else asm volatile("" : "+v"(pos[0]), "+v"(pos[1]));
        }
    };
    constexpr int LEAF0 = D >= STAGED_MIN_DEPTH ? 0 : (1 << D);  // what leaf4 / 4 counts from

    if constexpr (MODE == MODE_SCALAR) {
        // wave-uniform base of the current tree's leaf values, shifted so that what the walk ends
        // on indexes it directly; carried from tree to tree in scalar registers
        LeafBytes lv = (LeafBytes)(m.leaf_value + ((t_begin << D) - LEAF0));
        int t = t_begin, column = 0;
        int column_end = uniform(static_cast<int>(m.col_trees[0]));
        while (t < t_end) {
            while (column_end <= t) column_end += uniform(static_cast<int>(m.col_trees[++column]));
            const int run_end = column_end < t_end ? column_end : t_end;
            accu.begin_tree(column);
            float pending[R];
#pragma unroll
            for (int r = 0; r < R; ++r) pending[r] = 0.0f;
            for (; t < run_end; ++t, lv += sizeof(float) << D) {
                asm volatile("" : "+s"(lv));
                uint32_t leaf4[R];
                walk_tree(leaf4);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    accu.add_value(r, pending[r]);
                    pending[r] = *(LeafFloat)(lv + leaf4[r]);
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) accu.add_value(r, pending[r]);
        }
    } else {
        MetaPtr meta = (MetaPtr)m.tree;
        for (int t = t_begin; t < t_end; ++t) {
            const int caller_tree = meta[t].caller_tree;
            uint32_t leaf4[R];
            walk_tree(leaf4);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int leaf = (t << D) + static_cast<int>(leaf4[r] >> 2) - LEAF0;
                if (MODE == MODE_LEAVES) {
                    const int64_t row = row0 + r * TILE + lane;
                    if (row < n_rows) leaf_out[row * T + caller_tree] = m.leaf_node[leaf];
                } else {
                    accu.add(m, r, leaf);
                }
            }
        }
    }
}

// Register budget: the 28 hand-placed registers, 32, 64 or 128 pinned rank registers (NVR = 1, 2,
// 4: from v28, v64 resp. v32 on) and the compiler's working set leave room for 6, 4 resp. 3 waves
// per SIMD (80, 128 resp. 168 VGPRs; a seventh wave of the smallest kernel needs spills and
// measured no faster).
template <int D, int NVR>
__global__ __launch_bounds__(BLOCK, (NVR == 1 ? 6 : NVR == 2 ? 4 : 3)) void forest_rank_kernel(DevModel m, const float *__restrict__ X,
                                                            int64_t n_rows, float *scores,
                                                            int32_t *labels, int32_t *leaf_out)
{
    constexpr int R = 2;
    extern __shared__ __align__(16) char smem[];
    // The walk's tables come first, at addresses the compiler knows: 128 two-byte records and two
    // tables of 128 bytes (rank_trees_hand; depths 4 and more read them).
    uint8_t *walk_tables = reinterpret_cast<uint8_t *>(smem);
    constexpr int FRONT = WALK_TABLE_BYTES + WAVES * deep_bytes_per_wave(D);  // tables, then the waves' strips for deep trees
    uint32_t *rk = reinterpret_cast<uint32_t *>(smem + FRONT);  // [32 * NVR][64] packed ranks, then reused as:
    double *acc = reinterpret_cast<double *>(smem + FRONT);     // [WAVES][K][128] partial sums

    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * RROWS;

    if (D >= STAGED_MIN_DEPTH && threadIdx.x < 128) {
        // Depths 4..6: the records hold 4 x leaf ordinals.  Depths 7, 8: the first two tables cover
        // levels 0..4 and hold ordinals of level-5 subtrees, the third one the path through such a
        // subtree (4 x the leaf's ordinal inside it).
        constexpr bool WHOLE = D <= STAGED_MAX_DEPTH;
        constexpr int LOWER = WHOLE ? (D - 3 > 0 ? D - 3 : 0) : 2;   // levels below the top three
        constexpr int FIELD = (1 << LOWER) - 1;                     // bits of a lower subtree's field
        constexpr int DEEP = WHOLE ? 0 : D - 5;                     // levels of a level-5 subtree
        const int t = threadIdx.x, path = staged_path(t);
        walk_tables[2 * t] = static_cast<uint8_t>(STAGED_FIELDS_AT + FIELD * path);
        walk_tables[2 * t + 1] = static_cast<uint8_t>(WHOLE ? path * (4 << LOWER) : 4 * path);
        walk_tables[256 + t] = static_cast<uint8_t>((path >> (3 - LOWER)) * (WHOLE ? 4 : 1));
        walk_tables[384 + t] = static_cast<uint8_t>((path >> (3 - DEEP)) * 4);
    }

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
        rank_trees_hand<D, NVR, MODE_LEAVES>(m, x, accu, wave, lane, row0, n_rows, leaf_out, walk_tables);
        return;
    }
    if (m.leaf_width == 1) rank_trees_hand<D, NVR, MODE_SCALAR>(m, x, accu, wave, lane, row0, n_rows, nullptr, walk_tables);
    else rank_trees_hand<D, NVR, MODE_VECTOR>(m, x, accu, wave, lane, row0, n_rows, nullptr, walk_tables);
    accu.flush();
    __syncthreads();
    const int li = threadIdx.x;
    if (li < RROWS) finish_row(m, acc, RROWS, li, row0 + li, row0 + li < n_rows, scores, labels);
}

size_t rank_lds_bytes(const DevModel &m, int nvr)
{
    const size_t a = sizeof(double) * WAVES * m.n_outputs * RROWS;
    const size_t b = sizeof(uint32_t) * 32 * nvr * TILE;
    return WALK_TABLE_BYTES + static_cast<size_t>(WAVES) * deep_bytes_per_wave(m.kind) + (a > b ? a : b);
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
            // the walk's tables are read at literal LDS addresses from 0 on: the kernel's dynamic
            // LDS must begin there, i.e. the kernel must have no static LDS
            hipFuncAttributes attr;
            e = hipFuncGetAttributes(&attr, reinterpret_cast<const void *>(pick_rank(nvr, d)));
            if (e != hipSuccess) return e;
            if (attr.sharedSizeBytes != 0) return hipErrorInvalidConfiguration;
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
