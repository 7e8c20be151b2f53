// Register-bank kernel of the LDS rank family (gfx950): trees of any shape, large batches.
//
// Same exact rewrite of the comparison as the other rank kernels (rank(x) > j instead of
// !(x <= tau_j), two rows per 32-bit register, v_pk_fma_f16 with clamp; Section 4.3.1 applied to
// the input), arranged so that no comparison reads LDS and one write of the register index serves
// four rows.  Every internal node of every tree is still evaluated for every row (Section 3.1.2,
// Fig. 2 steps (1) and (2)); what changes is who evaluates it:
//
//   * A workgroup of 8 waves owns 256 rows, four per lane.  The rank registers (one per feature,
//     more for a feature with very many thresholds) are dealt to the waves, up to 32 each, and stay
//     in vector registers -- v64.. for the lane's rows l and l + 64, v96.. for rows l + 128 and
//     l + 192 -- selected by the VGPR index mode (step (1), matmul(X, W1), costs no vector
//     instruction, and one scalar instruction per node sets the index for both comparisons).
//   * The trees are taken 2 at a time (a batch).  Each wave evaluates the nodes of the batch that
//     test one of ITS registers -- a stream of entries the host compiler sorted that way, read 16
//     entries at a time into two alternating sets of scalar registers -- and the matrix core turns
//     every 8 outcomes into a byte per row, stored in an LDS buffer the whole workgroup shares.
//     A node's place in that buffer is its slot.
//   * After a barrier every lane walks one (row, tree) of the batch from the root: the outcome bit
//     of its slot and the slot's child references pick the next slot, until a leaf (the bit-level
//     form of matmul(., W3) + argmax).  A wave owns 32 of the workgroup's rows for all trees, so
//     the sums over trees never leave the wave: each of the 2 lanes of a row sums the trees it
//     walked, in fp64, and one cross-lane addition at the end joins them.
//
// Against the LDS-resident rank kernel this takes the LDS read per comparison (the LDS was the
// busiest unit there), half of the scalar instructions per comparison and the per-group
// bookkeeping of the level-by-level walk out of the evaluation loop.  The price is a barrier pair
// per batch and padding of every wave's share of a batch to whole units of 16 entries.  Small
// batches, and models whose batch buffer or registers do not fit, run the LDS-resident kernel.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"
#include "forest_kernel_common.hpp"
#include "forest_rank_common.hpp"

namespace forest_impl {
namespace {

constexpr int BANK_BLOCK = TILE * BANK_WAVES;
constexpr unsigned BANK_STAGGER_BLOCKS = 512;  // two workgroups on each of 256 compute units
constexpr int BANK_STAGGER_NAPS = 30;          // of 127 * 64 cycles: about 100 microseconds in all
constexpr int BANK_ROWS_PER_WAVE = BANK_ROWS / BANK_WAVES;  // rows a wave walks
static_assert(BANK_ROWS_PER_WAVE * BANK_TREES == TILE, "one lane per (row, tree) of a batch");
static_assert(BANK_ROWS == BANK_WAVES * 32 && BANK_PASS_FEATURES == 64, "the staging step: 16 lanes per row, 32 rows per step");
static_assert(BANK_REGS == 32 && BANK_ROWS == 4 * TILE, "the comparison statement addresses v64..v95 and v96..v127");
static_assert(BANK_UNIT == 16, "a unit is one 16-register scalar load: two groups of 8 entries");

#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) BankSpan *SpanPtr;
typedef const __attribute__((address_space(4))) BankBatch *BatchPtr;
typedef const __attribute__((address_space(4))) BankPass *PassPtr;
typedef const __attribute__((address_space(4))) BankPassWave *PassWavePtr;
typedef const __attribute__((address_space(4))) BankTodo *TodoPtr;
#else
typedef const BankSpan *SpanPtr;  // host pass: the kernel body is only parsed
typedef const BankBatch *BatchPtr;
typedef const BankPass *PassPtr;
typedef const BankPassWave *PassWavePtr;
typedef const BankTodo *TodoPtr;
#endif

enum { BANK_SUMS = 0, BANK_LEAVES = 1 };

// Eight entries applied to the lane's four rows: one index write, two comparisons per entry.
// The outcome registers are pinned (v48.., v56..) so that the statement can name them one by one
// and hand them to the matrix core as two 8-register operands.
#define FOREST_BANK_CMP(n, A, B)                                                              \
    "v_pk_fma_f16 " A ", v64, 4.0, %[e" #n "] op_sel:[0,0,1] op_sel_hi:[1,0,1] clamp\n\t"      \
    "v_pk_fma_f16 " B ", v96, 4.0, %[e" #n "] op_sel:[0,0,1] op_sel_hi:[1,0,1] clamp\n\t"
__device__ __forceinline__ void bank_compare(v8i &da, v8i &db, const Entry8 &q, const v32u &xa, const v32u &xb)
{
    asm volatile("s_set_gpr_idx_on %[e0], 0x1\n\t" FOREST_BANK_CMP(0, "v48", "v56")
                 "s_set_gpr_idx_idx %[e1]\n\t" FOREST_BANK_CMP(1, "v49", "v57")
                 "s_set_gpr_idx_idx %[e2]\n\t" FOREST_BANK_CMP(2, "v50", "v58")
                 "s_set_gpr_idx_idx %[e3]\n\t" FOREST_BANK_CMP(3, "v51", "v59")
                 "s_set_gpr_idx_idx %[e4]\n\t" FOREST_BANK_CMP(4, "v52", "v60")
                 "s_set_gpr_idx_idx %[e5]\n\t" FOREST_BANK_CMP(5, "v53", "v61")
                 "s_set_gpr_idx_idx %[e6]\n\t" FOREST_BANK_CMP(6, "v54", "v62")
                 "s_set_gpr_idx_idx %[e7]\n\t" FOREST_BANK_CMP(7, "v55", "v63")
                 "s_set_gpr_idx_off"
                 : "={v[48:55]}"(da), "={v[56:63]}"(db)
                 : [e0] "s"(q.e[0]), [e1] "s"(q.e[1]), [e2] "s"(q.e[2]), [e3] "s"(q.e[3]), [e4] "s"(q.e[4]),
                   [e5] "s"(q.e[5]), [e6] "s"(q.e[6]), [e7] "s"(q.e[7]), "{v[64:95]}"(xa), "{v[96:127]}"(xb));
}

// Register `slot` (wave-uniform) of the wave's bank takes `a` (rows l and l + 64 of the lane) and `b`
// (rows l + 128 and l + 192): a vector element written at a run-time index, which the compiler
// turns into the index mode applied to the destination.
__device__ __forceinline__ void bank_set(v32u &xa, v32u &xb, int slot, uint32_t a, uint32_t b)
{
    xa[slot] = a;
    xb[slot] = b;
}

// The ranks of the workgroup's rows, straight into the waves' banks.  X is read in blocks of up to
// BANK_PASS_FEATURES columns: every row's part of the block is contiguous in memory and goes to
// LDS as it lies there (16 bytes per lane, 16 lanes per row, each 128-byte line read once, by one
// wave, and not kept in the caches: the model's tables stay there instead); then every wave looks
// up the registers of its own bank that belong to the block -- all four rows of a lane for one
// register at a time, the feature's constants in scalar registers, the values read from LDS
// (a column of the block, rows across lanes, odd pitch), the table reads of the next register
// under way while the windows of this one are counted.
__device__ __forceinline__ void bank_ranks(const DevModel &m, const float *__restrict__ X, int64_t row0, int64_t n_rows,
                                           float *tile, v32u &xa, v32u &xb, int wave, int lane)
{
    const int F = m.n_features;
    PassPtr pass = (PassPtr)m.bank.pass;
    PassWavePtr pass_wave = (PassWavePtr)m.bank.pass_wave;
    TodoPtr todo = (TodoPtr)m.bank.todo;
    FastPtr feat = (FastPtr)m.fast_feat;
    const int piece = threadIdx.x & 15;      // which 16 bytes of a row's part of the block
    const int row_of_step = threadIdx.x >> 4;  // 32 rows per step
    for (int p = 0; p < m.bank.passes; ++p) {
        const int f_begin = pass[p].feat_begin, f_end = pass[p].feat_end;
        const int f_mine = f_begin + 4 * piece;
        if (f_mine < f_end) {
            typedef float Run4 __attribute__((ext_vector_type(4), aligned(4)));
            Run4 v[BANK_ROWS / 32];
#pragma unroll
            for (int s = 0; s < BANK_ROWS / 32; ++s) {
                const int64_t row = row0 + s * 32 + row_of_step;
                v[s] = Run4{0.0f, 0.0f, 0.0f, 0.0f};
                if (row < n_rows) {
                    const float *src = X + row * F + f_mine;
                    if (f_mine + 4 <= F) {
                        v[s] = __builtin_nontemporal_load(reinterpret_cast<const Run4 *>(src));
                    } else {  // the row ends inside the piece
#pragma unroll
                        for (int i = 0; i < 3; ++i)
                            if (f_mine + i < F) v[s][i] = src[i];
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < BANK_ROWS / 32; ++s) {
                float *dst = tile + (s * 32 + row_of_step) * BANK_TILE_PITCH + 4 * piece;
#pragma unroll
                for (int i = 0; i < 4; ++i) dst[i] = v[s][i];
            }
        }
        __syncthreads();  // the block is staged
        const BankPassWave pw = pass_wave[p * BANK_WAVES + wave];
        const float *mine = tile + lane * BANK_TILE_PITCH - f_begin;  // + feature: the lane's first row of that column
        if (pw.n_fast > 0) {
            BankTodo td = todo[pw.begin];
            FastLookup bf = feat[td.feature];
            auto begin = [&](const BankTodo &item, const FastLookup &ff) {
                const float *column = mine + item.feature;
                float xs[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) xs[j] = column[j * TILE * BANK_TILE_PITCH];
                return fast_lookup_begin<4>(m, ff, xs);
            };
            FastWindows<4> q = begin(td, bf);
            for (int k = 0; k < pw.n_fast; ++k) {
                // the next register's first half (the last one repeats itself; not used)
                const BankTodo td_next = todo[pw.begin + (k + 1 < pw.n_fast ? k + 1 : k)];
                const FastLookup bf_next = feat[td_next.feature];
                const FastWindows<4> q_next = begin(td_next, bf_next);
                int rank[4];
                fast_lookup_end<4, 2>(m, q, bf, td.feature, rank);
                bank_set(xa, xb, td.slot, fast_code_pair(rank[0], rank[1]), fast_code_pair(rank[2], rank[3]));
                td = td_next;
                bf = bf_next;
                q = q_next;
            }
        }
        for (int k = 0; k < pw.n_slow; ++k) {  // any number of thresholds, any register of the feature
            const BankTodo td = todo[pw.begin + pw.n_fast + k];
            uint32_t code[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int local = rank_of(m, td.feature, mine[td.feature + j * TILE * BANK_TILE_PITCH]) - td.first;
                local = local < 0 ? 0 : (local > td.len ? td.len : local);
                code[j] = rank_code_bits(local);
            }
            bank_set(xa, xb, td.slot, code[0] | (code[1] << 16), code[2] | (code[3] << 16));
        }
        __syncthreads();  // the block's place is free: for the next block, or for the outcome bytes
    }
}

// Makes whatever is computed from `p` afterwards wait for `set` to have arrived: the statement
// reads the set's first register and hands `p` back as a value the compiler knows nothing about.
__device__ __forceinline__ void issue_after(ProgPtr &p, const Batch<16> &set)
{
    asm volatile("" : "+s"(p) : "s"(set.q[0].e[0]));
}

// The row of the workgroup's tile that a lane walks: lanes 2 i and 2 i + 1 of wave w take row
// 8 i + w (one tree of the batch each).  A wave's 32 rows are 8 apart, so their outcome bytes of one
// group lie in 32 different LDS banks (rows next to each other would share 8 banks, and the walk's
// byte reads, which every lane makes at every step, would queue eight deep).
__device__ __forceinline__ int bank_walk_row(int wave, int lane)
{
    static_assert(BANK_ROWS_PER_WAVE * BANK_WAVES == BANK_ROWS, "every row of the tile is walked by one wave");
    return (lane / BANK_TREES) * BANK_WAVES + wave;
}

// The half of `pair` that the outcome bit of the slot at byte offset `at` picks (`byte`: the
// outcome byte of the slot's group): three bit-field extractions and a shift, no comparison and
// no select.
__device__ __forceinline__ uint32_t pick_half(uint32_t pair, uint32_t byte, uint32_t at)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const uint32_t bit = __builtin_amdgcn_ubfe(byte, __builtin_amdgcn_ubfe(at, 2u, 3u), 1u);
    return __builtin_amdgcn_ubfe(pair, bit << 4, 16u);
#else
    return ((byte >> ((at >> 2) & 7u)) & 1u) ? (pair >> 16) : (pair & 0xffffu);
#endif
}

// sum over the lanes that share a row (one per tree of the batch), the same bits in each
__device__ __forceinline__ double row_sum(double v)
{
    static_assert(BANK_TREES == 2, "one cross-lane addition");
    return v + __shfl_xor(v, 1);
}

// buf: the batch's outcome bytes ([group of 8 slots][row of the workgroup]); child_lds: the batch's
// child references, one word per slot.
template <int MODE>
__device__ __forceinline__ void bank_trees(const DevModel &m, const v32u &xa, const v32u &xb, uint8_t *buf,
                                           uint32_t *child_lds, double (&sum)[2], int wave, int lane, int64_t row0,
                                           int64_t n_rows, int32_t *leaf_out)
{
    const int T = m.n_trees;
    const int K = m.n_outputs;
    const int walk_row = bank_walk_row(wave, lane);                      // the lane's row of the tile in the walk
    const int walk_tree = lane % BANK_TREES;                            // and its tree of the batch
    const int64_t row = row0 + walk_row;
    BitCollector bits;
    bits.init(lane);
    ProgPtr p = (ProgPtr)(m.bank.prog + m.bank.stream_base[wave]);
    SpanPtr span = (SpanPtr)m.bank.span;
    BatchPtr batch = (BatchPtr)m.bank.batch;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    // The stream lives in two sets of 16 scalar registers used in turn: while one is evaluated
    // the other is being loaded.
    Batch<16> set_a = load_batch<16>(p), set_b = load_batch<16>(p + 16);
    // What a walk ends on is fetched at once and used a batch later (the gather's latency is
    // covered by the next batch's comparisons): the leaf's values, or, for the leaf-id output,
    // the caller's node index with the place it goes to.
    float pend_v0 = 0.0f, pend_v1 = 0.0f;
    int pend_node = 0, pend_tree = 0;
    bool pend_valid = false;
    auto consume_pending = [&]() {
        if (MODE == BANK_LEAVES) {
            if (pend_valid && row < n_rows) leaf_out[row * T + pend_tree] = pend_node;
        } else {
            // K == 1 (scalar leaves) or K == leaf width <= 2: the sums stay in registers, one per
            // lane (the trees the lane walked); the lanes of a row add theirs up at the end
            sum[0] += pend_valid ? static_cast<double>(pend_v0) : 0.0;
            if (K > 1) sum[1] += pend_valid ? static_cast<double>(pend_v1) : 0.0;
        }
    };

    // The records of a batch (the wave's span, the batch's slots and steps) are read a batch ahead:
    // read where they are needed, every batch would begin and end with a wait for a scalar load.
    BankSpan span_next = span[wave];
    BankBatch batch_next = batch[0];
    // Everything loaded so far has arrived before the first batch begins, as it has at the end of
    // every batch (the barrier's wait): the compiler then knows that the records requested at the
    // top of a batch are all that is on its way there, and does not wait for them before the
    // first comparisons.
    issue_after(p, set_a);
    issue_after(p, set_b);
    asm volatile("" : : "s"(span_next.n_units), "s"(batch_next.n_slots));
    for (int b = 0; b < m.bank.batches; ++b) {
        const BankSpan my_span = span_next;
        const BankBatch this_batch = batch_next;
        {
            const int nb = b + 1 < m.bank.batches ? b + 1 : b;
            span_next = span[nb * BANK_WAVES + wave];
            batch_next = batch[nb];
        }
        const int n_units = my_span.n_units;
        // The batch's child references go to LDS: the walk reads one per step and lane, which
        // the texture path serves at about one lane per cycle and the LDS far faster.  Four
        // words per thread, fetched now, stored after the evaluation.
        const int n_slots = this_batch.n_slots;
        const int tid = wave * TILE + lane;
        const bool stage = 4 * tid < n_slots;  // n_slots is a multiple of 16
        u32x4 staged = {0u, 0u, 0u, 0u};
        if (stage) staged = reinterpret_cast<const u32x4 *>(m.bank.child + this_batch.slot_base)[tid];
        const BankTree bt = m.bank.tree[b * BANK_TREES + walk_tree];  // used after the evaluation
        // `prev`: where the bytes of the lane's four rows go for the group BEFORE the first group of
        // the current pair of units (prev[0], prev[64], prev[128], prev[192]); the groups of the pair
        // are at prev + 256, + 512, ...  The buffer starts 256 bytes into the LDS, so `prev` is a
        // valid address for a wave's first group too (nothing is stored through it then).
        uint8_t *prev = buf + my_span.unit_base * (2 * BANK_ROWS) + lane - BANK_ROWS;
        // ---- evaluation: this wave's nodes of the batch.  A group's byte is still being
        // collected by the matrix core when its last comparison has issued, so it is stored
        // after the comparisons of the next group.
        v4f ga = bits.bias, gb = bits.bias;
        bool pending = false;
        auto store = [&](int k) {  // the bytes of group k - 1 of the pair (k = 0: the last one of the pair before)
            prev[k * BANK_ROWS] = static_cast<uint8_t>(__float_as_uint(ga[0]));
            prev[k * BANK_ROWS + TILE] = static_cast<uint8_t>(__float_as_uint(ga[1]));
            prev[k * BANK_ROWS + 2 * TILE] = static_cast<uint8_t>(__float_as_uint(gb[0]));
            prev[k * BANK_ROWS + 3 * TILE] = static_cast<uint8_t>(__float_as_uint(gb[1]));
        };
        // The same stores for a group whose bytes the matrix core finished long ago: inside the
        // loop a whole group of comparisons (26 instructions) lies between a matrix instruction and
        // the store of its result, more than the 11 wait states it needs.  The compiler cannot
        // count the instructions of the comparison statement and would pad every store with idle
        // cycles; written as a statement of their own the stores go out at once.
#if defined(__HIP_DEVICE_COMPILE__)
        typedef __attribute__((address_space(3))) uint8_t *LdsBytes;
#endif
        auto store_late = [&](int k) {
#if defined(__HIP_DEVICE_COMPILE__)
            const uint32_t to = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((LdsBytes)prev));
            asm volatile("ds_write_b8 %0, %1 offset:%5\n\t"
                         "ds_write_b8 %0, %2 offset:%6\n\t"
                         "ds_write_b8 %0, %3 offset:%7\n\t"
                         "ds_write_b8 %0, %4 offset:%8"
                         :
                         : "v"(to), "v"(ga[0]), "v"(ga[1]), "v"(gb[0]), "v"(gb[1]), "n"(k * BANK_ROWS),
                           "n"(k * BANK_ROWS + TILE), "n"(k * BANK_ROWS + 2 * TILE), "n"(k * BANK_ROWS + 3 * TILE)
                         : "memory");
#endif
        };
        // One group: its comparisons, then the stores of the group before, then its bytes' turn on
        // the matrix core.  `between` runs after the comparisons (k: constant at every call).
        auto group = [&](const Entry8 &q, int k, auto between) {
            v8i da, db;
            bank_compare(da, db, q, xa, xb);
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_sched_barrier(0);
#endif
            between();
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_sched_barrier(0);
#endif
            if (pending) store_late(k);
#if defined(__HIP_DEVICE_COMPILE__)
            __builtin_amdgcn_sched_barrier(0);
#endif
            ga = bits.collect_b(da, bits.bias);
            gb = bits.collect_b(db, bits.bias);
            pending = true;
        };
        auto nothing = [] {};
        // The stream: set_a holds the unit evaluated next and has arrived, set_b the unit after it
        // and is on its way (a wave's units follow each other from batch to batch, so this holds
        // from one batch to the next).  Scalar loads may return out of order and share their counter
        // with the LDS, so a wait for one is a wait for everything: the wait for the set on its
        // way sits after the comparisons of a unit's second group -- the load has had most of two
        // groups to arrive, the last stores a whole group -- and the set just used up is loaded
        // again right behind it, tied to the wait through the stream pointer.
        // While it evaluates, the wave goes first among the waves of its SIMD: the walks and lookups
        // of the others are chains of waits that fill whatever issue slots it leaves (1 % on c5).
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_s_setprio(3);
#endif
        int u = 0;
        for (; u + 1 < n_units; u += 2) {
            group(set_a.q[0], 0, nothing);
            group(set_a.q[1], 1, [&] {
                issue_after(p, set_b);
                set_a = load_batch<16>(p + 32);
            });
            group(set_b.q[0], 2, nothing);
            group(set_b.q[1], 3, [&] {
                issue_after(p, set_a);
                set_b = load_batch<16>(p + 48);
            });
            p += 32;
            prev += 4 * BANK_ROWS;
        }
        if (u < n_units) {
            group(set_a.q[0], 0, nothing);
            group(set_a.q[1], 1, [&] {
                issue_after(p, set_b);
                set_a = set_b;
                set_b = load_batch<16>(p + 32);
            });
            p += 16;
            prev += 2 * BANK_ROWS;
        }
#if defined(__HIP_DEVICE_COMPILE__)
        __builtin_amdgcn_s_setprio(0);
#endif
        if (pending) store(0);  // right behind its matrix instructions: the compiler's own store, with the wait
        if (stage) reinterpret_cast<u32x4 *>(child_lds)[tid] = staged;
        if (b > 0) consume_pending();  // the last batch's leaves
#if defined(__HIP_DEVICE_COMPILE__)
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the loop's stores are not the compiler's to wait for
#endif
        __syncthreads();  // the batch's bits and child references are complete

        // ---- walk: one (row, tree) per lane.  Every lane takes the batch's number of steps: a step
        // reads the outcome byte and the word of where the lane stands (both reads in flight
        // together) and moves to the half of the word the outcome bit picks, which is the same
        // place again once the next node would be a leaf; no test, no branch but the loop's.
        // Both reads at literal LDS addresses (the kernel has no static LDS, so its dynamic LDS
        // begins at address 0; init_rankbank_kernels checks that): a slot's word at the constant
        // place of the child table plus the slot's offset, its group's byte at 256 bytes per
        // group from the row's byte of group 0.
#if defined(__HIP_DEVICE_COMPILE__)
        typedef const __attribute__((address_space(3))) uint8_t *LdsByte;
        typedef const __attribute__((address_space(3))) uint32_t *LdsWord;
        const uint32_t row_byte = static_cast<uint32_t>(BANK_ROWS + sizeof(uint32_t) * BANK_UNIT * m.bank.max_units) + static_cast<uint32_t>(walk_row);
        auto outcome_byte = [&](uint32_t where) -> uint32_t {
            uint32_t group = where >> 5;
            asm volatile("" : "+v"(group));  // keeps shift and shift-and-add apart: two instructions, not three
            return *(LdsByte)static_cast<uintptr_t>(row_byte + (group << 8));
        };
        auto child_word = [&](uint32_t where) -> uint32_t { return *(LdsWord)static_cast<uintptr_t>(BANK_ROWS + where); };
#else
        const uint8_t *bits_of_row = buf + walk_row;  // host pass: the kernel body is only parsed
        auto outcome_byte = [&](uint32_t where) -> uint32_t { return bits_of_row[(where >> 5) << 8]; };
        auto child_word = [&](uint32_t where) -> uint32_t { return child_lds[where >> 2]; };
#endif
        const bool single_leaf = (static_cast<uint32_t>(bt.root_ref) & BANK_LEAF_FLAG) != 0u;
        uint32_t at = single_leaf ? 0u : static_cast<uint32_t>(bt.root_ref);  // byte offset of the slot's word
        const int steps = this_batch.steps;
        auto move = [&] {
            const uint32_t byte = outcome_byte(at);  // group (at / 32) of BANK_ROWS bytes
            const uint32_t c = child_word(at);
            at = pick_half(c, byte, at);
        };
        int step = 0;
        for (; step + 4 <= steps; step += 4) {  // (written out: the statement in outcome_byte keeps the compiler from unrolling)
            move();
            move();
            move();
            move();
        }
        for (; step < steps; ++step) move();
        // where the lane stands now, the outcome bit picks a leaf
        const uint32_t last_byte = outcome_byte(at);
        const uint32_t leaves = m.bank.leaf[this_batch.slot_base + (at >> 2)];
        const uint32_t picked = pick_half(leaves, last_byte, at);
        // index into the per-leaf tables; the record that fills a batch of one tree gives leaf 0
        const int leaf = bt.leaf_base + static_cast<int>(single_leaf ? 0u : picked);
        pend_valid = bt.valid != 0;
        if (MODE == BANK_LEAVES) {
            pend_node = m.leaf_node[leaf];
            pend_tree = bt.caller_tree;
        } else {
            const float *v = m.leaf_value + static_cast<size_t>(leaf) * K;
            pend_v0 = v[0];
            if (K > 1) pend_v1 = v[1];
        }
        __syncthreads();  // every lane is done with the buffer
    }
    if (m.bank.batches > 0) consume_pending();
}

// 128 vector registers per lane at most: two workgroups of 8 waves per compute unit.
template <int MODE>
__global__ __launch_bounds__(BANK_BLOCK) __attribute__((amdgpu_waves_per_eu(4, 4))) void forest_rankbank_kernel(
    DevModel m, const float *__restrict__ X, int64_t n_rows, float *scores, int32_t *labels, int32_t *leaf_out,
    int stagger)
{
    extern __shared__ __align__(16) char smem[];
    // Workgroups all take the same time, so those that start together read their rows of X together,
    // round after round, and wait for memory together.  The workgroups of the first round (the
    // ones resident at once) start up to `stagger` sleeps apart instead, which spreads the reads
    // of every later round as well.  A bounded wait: nothing is waited FOR.
    if (blockIdx.x < BANK_STAGGER_BLOCKS) {
        const int naps = static_cast<int>((blockIdx.x * 40503u) % BANK_STAGGER_BLOCKS) * stagger / BANK_STAGGER_BLOCKS;
        for (int i = 0; i < naps; ++i) __builtin_amdgcn_s_sleep(127);
    }
    // LDS: first a block of X for the rank lookups ([row of the workgroup][column of the block], odd
    // pitch), then, in the same place, the batch's outcome bytes ([group of 8 slots][row of the
    // workgroup]) and child references.
    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * BANK_ROWS;

    v32u xa, xb;
#pragma unroll
    for (int i = 0; i < BANK_REGS; ++i) xa[i] = xb[i] = 0;  // registers the bank does not use stay defined
    bank_ranks(m, X, row0, n_rows, reinterpret_cast<float *>(smem), xa, xb, wave, lane);
    // From here on the lane's index is counted anew (two instructions) wherever it is needed: kept
    // in a register across the prologue, whose every register is spoken for, it would be spilled.
#if defined(__HIP_DEVICE_COMPILE__)
    const int lane_now = static_cast<int>(__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)));
#else
    const int lane_now = lane;
#endif

    double sum[2] = {0.0, 0.0};
    // a row of spare bytes, the batch's child references at a place the compiler knows (the walk
    // then reads a slot's word at the slot's offset plus a constant, no addition), the outcome
    // bytes behind them (`prev` in bank_trees may point one group in front of them)
    uint32_t *child_lds = reinterpret_cast<uint32_t *>(smem + BANK_ROWS);
    uint8_t *buf = reinterpret_cast<uint8_t *>(child_lds) + sizeof(uint32_t) * BANK_UNIT * static_cast<size_t>(m.bank.max_units);
    bank_trees<MODE>(m, xa, xb, buf, child_lds, sum, wave, lane_now, row0, n_rows, leaf_out);
    if (MODE == BANK_LEAVES) return;
    const int64_t row = row0 + bank_walk_row(wave, lane_now);
    // a copy with run-time indices: indexed that way `sum` itself would live in scratch memory
    double raw[2] = {row_sum(sum[0]), row_sum(sum[1])};
    if (lane_now % BANK_TREES == 0 && row < n_rows) finish_values(m, raw, 1, row, scores, labels);
}

size_t rankbank_lds_bytes(const DevModel &m)
{
    const size_t tile = sizeof(float) * BANK_ROWS * BANK_TILE_PITCH;
    // a row of spare bytes, a batch's child references (a word per slot), then its outcome bytes
    const size_t bytes = BANK_ROWS + (static_cast<size_t>(BANK_ROWS) * (BANK_UNIT / 8) + sizeof(uint32_t) * BANK_UNIT) *
                                         static_cast<size_t>(m.bank.max_units);
    return tile > bytes ? tile : bytes;
}

}  // namespace

hipError_t init_rankbank_kernels(size_t lds_limit)
{
    for (const void *fn : {reinterpret_cast<const void *>(forest_rankbank_kernel<BANK_SUMS>),
                           reinterpret_cast<const void *>(forest_rankbank_kernel<BANK_LEAVES>)}) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_limit));
        if (e != hipSuccess) return e;
        // the walk reads LDS at literal addresses from 0 on: the kernel's dynamic LDS must begin
        // there, i.e. the kernel must have no static LDS
        hipFuncAttributes attr;
        e = hipFuncGetAttributes(&attr, fn);
        if (e != hipSuccess) return e;
        if (attr.sharedSizeBytes != 0) return hipErrorInvalidConfiguration;
    }
    return hipSuccess;
}

hipError_t launch_rankbank(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                           int32_t *leaf_out, size_t lds_limit, hipStream_t stream)
{
    // what the kernel assumes of the model, checked before it runs
    const int K = m.n_outputs, W = m.leaf_width;
    const bool sums_fit = (K == 1 && W == 1) || (W == K && K <= 2);
    const size_t lds = rankbank_lds_bytes(m);
    if (!m.bank.enabled || m.n_splits != 1 || !sums_fit || m.rank_regs < 1 || m.rank_regs > BANK_WAVES * BANK_REGS || m.bank.passes < 1 ||
        lds > lds_limit || lds > BANK_MAX_LDS)
        return hipErrorInvalidValue;
    const int64_t n_blocks = (n_rows + BANK_ROWS - 1) / BANK_ROWS;
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(n_blocks));
    // only where the launch runs for many rounds: a short one would just start late
    const int stagger = n_blocks >= 8 * static_cast<int64_t>(BANK_STAGGER_BLOCKS) ? BANK_STAGGER_NAPS : 0;
    if (leaf_out)
        hipLaunchKernelGGL(forest_rankbank_kernel<BANK_LEAVES>, grid, dim3(BANK_BLOCK), lds, stream, m, X, n_rows,
                           scores, labels, leaf_out, stagger);
    else
        hipLaunchKernelGGL(forest_rankbank_kernel<BANK_SUMS>, grid, dim3(BANK_BLOCK), lds, stream, m, X, n_rows,
                           scores, labels, leaf_out, stagger);
    return hipGetLastError();
}

}  // namespace forest_impl
