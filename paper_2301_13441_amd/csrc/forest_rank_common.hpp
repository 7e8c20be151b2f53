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

// Bit collection on the matrix core.  The eight outcome registers of a group are, read as
// bytes, (0, a, 0, b) with a, b = 0x3c or 0 for the lane's two rows; 0x3c is 1.0 in bf8
// (e5m2).  v_mfma_f32_16x16x128_f8f6f4 takes them as its B operand: a lane of 16-lane block q
// supplies B[k][n] for n = lane % 16 and the 32 values of k that belong to block q, and
// receives D[4q + i][n], i = 0..3.  With an A that is zero outside A[4q + i][k of block q],
// D[4q + i][n] only sums the lane's own bytes: i = 0 weighs the row-a bytes by 2^(7 - v)
// (register v of the group: first entry in bit 7), i = 1 the row-b bytes.  On top of a 2^23
// addend the MFMA therefore leaves the 8 outcome bits of a group in the low mantissa bits of
// D[..][0] and D[..][1]: exact, every product and partial sum being an integer below 2^24.  The
// matrix core runs beside the vector ALU, so collecting a group costs the vector ALU the MFMA's
// issue instead of the eight instructions of a packed fused-multiply-add tree.
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct BitCollector {
    v8i a;  // weights 2^(7 - v)
    v4f bias;

    __device__ __forceinline__ void init(int lane)
    {
        const int m = lane & 15, q = lane >> 4;
        const bool mine = (m >> 2) == q && (m & 3) < 2;
        const int shift = (m & 3) == 0 ? 8 : 24;  // byte 1 = row a, byte 3 = row b
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const uint32_t bf8 = static_cast<uint32_t>(15 + 7 - v) << 2;  // 2^(7 - v) in e5m2
            a[v] = mine ? static_cast<int>(bf8 << shift) : 0;
        }
        bias = v4f{8388608.0f, 8388608.0f, 8388608.0f, 8388608.0f};
        // keep the addend in registers instead of rebuilding it before every chain
        asm volatile("" : "+v"(bias));
    }
    // the eight outcome registers of a group, in one tuple
    __device__ __forceinline__ v4f collect_b(const v8i &b, v4f c) const
    {
#if defined(__HIP_DEVICE_COMPILE__)
        c = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 1, 1, 0, 0, 0, 0);  // A, B: bf8, unscaled
        __builtin_amdgcn_sched_barrier(0);
#endif
        return c;
    }
};

#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) int32_t *RankTablePtr;
typedef const __attribute__((address_space(4))) FeatBucket *BucketPtr;
#else
typedef const int32_t *RankTablePtr;  // host pass: the kernel body is only parsed
typedef const FeatBucket *BucketPtr;
#endif

// bucket_index without branches: the same value for every x (maximum and minimum drop a NaN
// operand, the conversion truncates), three vector instructions after the subtraction and the
// multiplication.  n_buckets is at most 2^20, exact in float.
__device__ __forceinline__ int32_t bucket_index_fast(float x, float lo, float scale, int32_t n_buckets)
{
    const float t = (x - lo) * scale;
    return static_cast<int32_t>(fminf(fmaxf(t, 0.0f), static_cast<float>(n_buckets - 1)));
}

// Bracket of rank(x) from the feature's bucket table; every candidate in [lo, hi] is a rank.
struct RankBracket {
    int lo, hi;
};

__device__ __forceinline__ RankBracket bucket_bracket(const FeatBucket &fb, const int32_t *__restrict__ start, float x)
{
    const int32_t *s = start + fb.start_base + bucket_index(x, fb.lo, fb.scale, fb.n_buckets);
    return RankBracket{s[0], s[1]};
}

// Whether [lo, hi] really brackets rank(x) = #{i : thr[i] < x} in the n sorted thresholds.  It
// does whenever the table was built with the arithmetic bucket_index runs here; checking it
// against the thresholds makes the result independent of that.
__device__ __forceinline__ bool bracket_holds(const float *__restrict__ thr, int n, RankBracket b, float x)
{
    // Both neighbours are read whatever the bracket is (indices clamped into the feature's
    // thresholds; the table has one spare element, so index 0 exists for a feature without
    // thresholds too): loads that do not hang on a condition can be in flight together.
    const int last = n > 0 ? n - 1 : 0;
    const int il = b.lo > 0 ? b.lo - 1 : 0;
    const int ih = b.hi < last ? b.hi : last;
    const float tl = thr[il], th = thr[ih];
    const bool below = (b.lo == 0) | (tl < x);
    const bool above = (b.hi == n) | !(th < x);
    return below & above;
}

// One lane, one (row, feature): the rank of x among the feature's thresholds (all for NaN).
__device__ __forceinline__ int rank_of(const DevModel &m, int f, float x)
{
    const int tb = m.feat_thr_base[f];
    const int n = m.feat_thr_base[f + 1] - tb;
    if (x != x) return n;  // NaN is right of every threshold
    const float *__restrict__ thr = m.thr_sorted + tb;
    RankBracket b = bucket_bracket(m.feat_bucket[f], m.bucket_start, x);
    if (!bracket_holds(thr, n, b, x)) b = RankBracket{0, n};
    while (b.lo < b.hi) {
        const int mid = (b.lo + b.hi) >> 1;
        if (thr[mid] < x) b.lo = mid + 1;
        else b.hi = mid;
    }
    return b.lo;
}

// Writes the rank of tile row r for feature f into the packed tile: one f16 per rank register of
// the feature; tile row r lives in lane r % 64, low half for r < 64, high half above.
__device__ __forceinline__ void store_rank(uint16_t *tile16, const DevModel &m, int f, int r, int rank)
{
    const int n = m.feat_thr_base[f + 1] - m.feat_thr_base[f];
    const int reg0 = m.feat_vfirst[f];
    for (int sgm = 0, first = 0; first < n; ++sgm, first += RANK_SEG) {
        const int len = n - first < RANK_SEG ? n - first : RANK_SEG;
        int rv = rank - first;
        rv = rv < 0 ? 0 : (rv > len ? len : rv);
        tile16[((reg0 + sgm) * TILE + (r & (TILE - 1))) * 2 + (r >> 6)] = rank_code_bits(rv);
    }
}

// Ranks of a tile with few valid rows (the tail of a batch): the (row, feature) pairs are dealt
// to the threads, so the searches of one row run side by side instead of one feature after the
// other; the rest of the tile gets rank 0.  Xt points at the tile's first row.
template <int NWAVES>
__device__ __forceinline__ void rank_rows_few(uint32_t *rk, const DevModel &m, const float *__restrict__ Xt,
                                              int n_valid, int f_begin, int f_end, int reg_begin, int reg_end)
{
    const int F = m.n_features;
    const int n_threads = NWAVES * TILE;
    for (int i = threadIdx.x; i < (reg_end - reg_begin) * TILE; i += n_threads) rk[i] = 0;
    __syncthreads();
    uint16_t *rk16 = reinterpret_cast<uint16_t *>(rk) - static_cast<ptrdiff_t>(reg_begin) * TILE * 2;
    const int nf = f_end - f_begin;
    for (int w = threadIdx.x; w < n_valid * nf; w += n_threads) {
        const int r = w / nf, f = f_begin + (w - r * nf);
        store_rank(rk16, m, f, r, rank_of(m, f, Xt[r * F + f]));
    }
}

// Split launches: the tile's ranks were computed by forest_rank_tiles_kernel; copy them from
// global memory into the LDS tile (coalesced, n_threads threads).
__device__ __forceinline__ void load_rank_tile(uint32_t *rk, const DevModel &m, int n_threads)
{
    const int words = m.rank_regs * TILE;
    const uint32_t *__restrict__ src = m.rank_tiles + static_cast<size_t>(blockIdx.x) * words;
    for (int i = threadIdx.x; i < words; i += n_threads) rk[i] = src[i];
}

// A table element at a wave-uniform base plus a per-lane 32-bit byte offset: the load takes the
// base from scalar registers and one vector register for the offset (the tables are far below
// 4 GB), instead of a 64-bit address built on the vector ALU.
template <typename T>
__device__ __forceinline__ T load_at(const void *__restrict__ base, uint32_t byte_offset)
{
    return *reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + byte_offset);
}

// N floats read with one load; the tables are only known to be 4-byte aligned.
template <int N>
struct __attribute__((aligned(4))) FloatRun {
    float v[N];
};

// ---------------------------------------------------------------------------------------
// The fast lookup (forest_model.hpp: FastLookup), N values of one feature per lane.
// ---------------------------------------------------------------------------------------
#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) FastLookup *FastPtr;
#else
typedef const FastLookup *FastPtr;  // host pass: the kernel body is only parsed
#endif

// The lane's N values of one feature, and where their windows begin.
template <int N>
struct FastWindows {
    float x[N];
    uint32_t at[N];  // byte offset of the window in the feature's thresholds
};

// First half: the values' buckets, and the table entries on their way (a window begins at the
// last threshold of the lower buckets, or where FAST_WINDOW thresholds still fit).
template <int N>
__device__ __forceinline__ FastWindows<N> fast_lookup_begin(const DevModel &m, const FastLookup &ff, const float (&x)[N])
{
    FastWindows<N> q;
    const char *tab = reinterpret_cast<const char *>(m.fast_tab) + ff.tab_off;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        q.x[j] = x[j];
        const float t = fminf(fmaxf((x[j] - ff.lo) * ff.scale, 0.0f), ff.last_bucket);  // NaN: bucket 0
        const uint32_t bucket = static_cast<uint32_t>(static_cast<int32_t>(t));
        q.at[j] = static_cast<uint32_t>(load_at<uint16_t>(tab, bucket << 1)) << 2;
    }
    return q;
}

// Second half: rank(x) = #{i : thr[i] < x} from the window thr[w .. w + FAST_WINDOW): w plus the
// number of its thresholds below x, provided every threshold before the window is below x (the
// window starts the list, or its first threshold is below x) and none after it is (it ends the
// list, or its last threshold is not below x).  The check is against the thresholds themselves;
// whatever it does not settle (a bucket fuller than a window, NaN) takes the general lookup.
// The windows are read G at a time (8 registers each).
template <int N, int G>
__device__ __forceinline__ void fast_lookup_end(const DevModel &m, const FastWindows<N> &q, const FastLookup &ff,
                                                int feature, int (&rank)[N])
{
    static_assert(N % G == 0, "whole groups of windows");
    const char *thr = reinterpret_cast<const char *>(m.thr_sorted) + ff.thr_off;
    const uint32_t last_at = static_cast<uint32_t>(ff.n - FAST_WINDOW) << 2;
    bool open[N];
    bool any_open = false;
#pragma unroll
    for (int h = 0; h < N; h += G) {
        FloatRun<FAST_WINDOW> w[G];
#pragma unroll
        for (int j = 0; j < G; ++j) w[j] = load_at<FloatRun<FAST_WINDOW>>(thr, q.at[h + j]);
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const float x = q.x[h + j];
            int count = 0;
#pragma unroll
            for (int i = 0; i < FAST_WINDOW; ++i) count += (w[j].v[i] < x) ? 1 : 0;
            const bool first_below = w[j].v[0] < x, last_below = w[j].v[FAST_WINDOW - 1] < x;
            open[h + j] = (!first_below & (q.at[h + j] != 0u)) | (last_below & (q.at[h + j] != last_at)) | (x != x);
            any_open |= open[h + j];
            rank[h + j] = static_cast<int>(q.at[h + j] >> 2) + count;
        }
    }
    if (__any(any_open)) {
#pragma unroll
        for (int j = 0; j < N; ++j)
            if (open[j]) rank[j] = rank_of(m, feature, q.x[j]);
    }
}

// Two ranks of a feature with a fast lookup as the packed codes of a rank register: such a feature
// has at most FAST_MAX_THRESHOLDS thresholds, all in one register, and every rank in the lower
// half of the codes, where code(q) = 0xf3ff - q.
__device__ __forceinline__ uint32_t fast_code_pair(int rank_lo, int rank_hi)
{
    constexpr uint32_t CODE0 = 0x8000u | (0x5c00u + RANK_CODES / 2 - 1);  // code(0)
    return (CODE0 - static_cast<uint32_t>(rank_lo)) | ((CODE0 - static_cast<uint32_t>(rank_hi)) << 16);
}

// Ranks of rows [row0, row0 + 128) for every feature with thresholds, written as packed f16
// pairs into rk[reg * 64 + lane] (low half: row `lane` of the tile, high half: row lane + 64).
// The features are dealt to the waves; inside a wave every lane looks up the same feature for
// its own two rows, U features at a time (2 U lookups in flight per lane), so the feature's
// constants are read with scalar loads.  A lookup is a bucket (a subtraction, a multiplication,
// a conversion), the bucket's lower bound of the rank from the start table, and a count over a
// window of 8 thresholds placed by that bound (or a binary search where the window does not
// decide the rank).  The lookups are bound by the rate at which the texture path takes per-lane
// addresses, so what counts is the number of reads per lookup: one table word and one window.
//
// The general form takes the features [f_begin, f_end), whose rank registers are
// [reg_begin, reg_end), and writes register r to rk[(r - reg_begin) * 64 + lane]: a tile of a
// part of the registers, for kernels that take the ranks out of LDS in several passes.
template <int NWAVES, int U = 2, bool STREAM_X = false>
__device__ __forceinline__ void rank_rows(uint32_t *rk, const DevModel &m, const float *__restrict__ X,
                                          int64_t row0, int64_t n_rows, int wave, int lane, int f_begin, int f_end,
                                          int reg_begin, int reg_end)
{
    const int F = m.n_features;
    const int64_t left = n_rows - row0;
    if (left * 4 <= RROWS) {  // workgroup-uniform
        rank_rows_few<NWAVES>(rk, m, X + row0 * F, static_cast<int>(left), f_begin, f_end, reg_begin, reg_end);
        return;
    }
    RankTablePtr thr_base = (RankTablePtr)m.feat_thr_base;
    RankTablePtr vfirst = (RankTablePtr)m.feat_vfirst;
    BucketPtr buckets = (BucketPtr)m.feat_bucket;
    const float *xrow[2];
    bool have[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int64_t row = row0 + r * TILE + lane;
        have[r] = row < n_rows;
        xrow[r] = X + (have[r] ? row : row0) * F;
    }
    for (int f0 = f_begin + wave * U; f0 < f_end; f0 += NWAVES * U) {
        float x[U][2];
        RankBracket b[U][2];
        int tb[U], n_thr[U];
        FeatBucket fb[U];
        // all feature values first, then all bucket reads: the loads of one kind go out together
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int f = f0 + u < f_end ? f0 + u : f_end - 1;  // wave-uniform; the duplicate is not stored
            tb[u] = thr_base[f];
            n_thr[u] = thr_base[f + 1] - tb[u];
            fb[u].lo = buckets[f].lo;
            fb[u].scale = buckets[f].scale;
            fb[u].n_buckets = buckets[f].n_buckets;
            fb[u].start_base = buckets[f].start_base;
            if (f0 + U > f_end) {
#pragma unroll
                for (int r = 0; r < 2; ++r)
                    x[u][r] = xrow[r][f];  // a row past the batch reads the tile's first row; its rank is not used
            }
        }
        if (f0 + U <= f_end) {  // wave-uniform: the U neighbouring features of a row in one load
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                // STREAM_X: a non-temporal load, so that X, read once, does not push the model's
                // tables out of the L2.  Only where the waves of a workgroup use up a 128-byte
                // line within an iteration or two; else the line would be fetched again.
                typedef float XRun __attribute__((ext_vector_type(U), aligned(4)));
                const XRun *p = reinterpret_cast<const XRun *>(xrow[r] + f0);
                const XRun v = STREAM_X ? __builtin_nontemporal_load(p) : *p;
#pragma unroll
                for (int u = 0; u < U; ++u) x[u][r] = v[u];
            }
        }
        // All U features with a fast lookup (wave-uniform; the usual case): table entry, window,
        // count -- a third of the instructions of the general lookup below.
        {
            FastPtr fast = (FastPtr)m.fast_feat;
            bool all_fast = f0 + U <= f_end;
#pragma unroll
            for (int u = 0; u < U; ++u) all_fast &= fast[f0 + u < f_end ? f0 + u : f_end - 1].fast != 0;
            if (all_fast) {
                FastLookup ff[U];
                FastWindows<2> q[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    ff[u] = fast[f0 + u];
                    q[u] = fast_lookup_begin<2>(m, ff[u], x[u]);
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    int rank[2];
                    fast_lookup_end<2, 2>(m, q[u], ff[u], f0 + u, rank);
                    rk[(vfirst[f0 + u] - reg_begin) * TILE + lane] = fast_code_pair(rank[0], rank[1]);
                }
                continue;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                // a feature with 8 thresholds or more only uses the lower end of the bracket
                if (n_thr[u] >= 8) {
                    const int32_t *st = m.bucket_start + fb[u].start_base;
                    b[u][r].lo = st[bucket_index_fast(x[u][r], fb[u].lo, fb[u].scale, fb[u].n_buckets)];
                    b[u][r].hi = n_thr[u];
                } else {
                    b[u][r] = bucket_bracket(fb[u], m.bucket_start, x[u][r]);
                }
            }
        // The rank from the bracket.  A feature with 8 thresholds or more (wave-uniform) reads one
        // window of 8 thresholds, thr[wb .. wb + 8) with wb = clamp(lo - 1, 0, n - 8), and counts those
        // below x: rank = wb + count, provided the window decides it -- every threshold before the
        // window is below x (the window starts at 0, or its first threshold already is below x) and
        // every threshold after it is not (some threshold of the window is not below x, or the
        // window ends the list).  That holds whenever the bucket's lower bound is within 6 of the
        // rank; it costs one table read and one window per lookup, and nothing of it rests on the
        // table having been built with the arithmetic bucket_index runs here.  What the window does
        // not decide, and features with fewer thresholds, go through the binary search below.
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float *thr = m.thr_sorted + tb[u];
            const int n = n_thr[u];
            if (n >= 8) {
                FloatRun<8> w[2];
                int wb[2];
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const int lo = b[u][r].lo - 1;
                    wb[r] = lo < 0 ? 0 : (lo > n - 8 ? n - 8 : lo);
                    w[r] = load_at<FloatRun<8>>(thr, static_cast<uint32_t>(wb[r]) << 2);
                }
                bool above[2];  // the whole window is below x and thresholds follow it: look further up
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const float xv = x[u][r];
                    int count = 0;
#pragma unroll
                    for (int i = 0; i < 8; ++i) count += (w[r].v[i] < xv) ? 1 : 0;
                    const bool closed = ((wb[r] == 0) | (count >= 1)) & ((count < 8) | (wb[r] + 8 >= n));
                    above[r] = (count == 8) & (wb[r] + 8 < n);
                    b[u][r].lo = closed ? wb[r] + count : 0;
                    b[u][r].hi = closed ? wb[r] + count : n;
                }
                // A bucket of a dense region can hold more thresholds than a window: slide the
                // window up, for the lanes concerned only (the reads of the others are masked off),
                // a few times before the search below takes over.
                for (int round = 0; round < 3 && __any(above[0] | above[1]); ++round) {
#pragma unroll
                    for (int r = 0; r < 2; ++r) {
                        if (above[r]) {
                            wb[r] = wb[r] + 7 > n - 8 ? n - 8 : wb[r] + 7;
                            const FloatRun<8> v = load_at<FloatRun<8>>(thr, static_cast<uint32_t>(wb[r]) << 2);
                            const float xv = x[u][r];
                            int count = 0;
#pragma unroll
                            for (int i = 0; i < 8; ++i) count += (v.v[i] < xv) ? 1 : 0;
                            // the window's first threshold is below x here (it was in the last window)
                            const bool closed = (count < 8) | (wb[r] + 8 >= n);
                            above[r] = !closed;
                            b[u][r].lo = closed ? wb[r] + count : 0;
                            b[u][r].hi = closed ? wb[r] + count : n;
                        }
                    }
                }
            } else {
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const bool ok = bracket_holds(thr, n, b[u][r], x[u][r]);
                    b[u][r].lo = ok ? b[u][r].lo : 0;
                    b[u][r].hi = ok ? b[u][r].hi : n;
                }
            }
        }
        // binary search inside the brackets: every step reads one threshold per lookup, whether
        // the lookup is still open or not (index clamped), so the four loads go out together
        for (;;) {
            bool more = false;
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < 2; ++r) more |= b[u][r].lo < b[u][r].hi;
            if (!more) break;
            float t[U][2];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const int last = n_thr[u] > 0 ? n_thr[u] - 1 : 0;
                    const int mid = (b[u][r].lo + b[u][r].hi) >> 1;
                    t[u][r] = m.thr_sorted[tb[u] + (mid < last ? mid : last)];
                }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const bool open = b[u][r].lo < b[u][r].hi;
                    const int mid = (b[u][r].lo + b[u][r].hi) >> 1;
                    const bool right = t[u][r] < x[u][r];
                    b[u][r].lo = (open & right) ? mid + 1 : b[u][r].lo;
                    b[u][r].hi = (open & !right) ? mid : b[u][r].hi;
                }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (f0 + u >= f_end) continue;
            int rank[2];
#pragma unroll
            for (int r = 0; r < 2; ++r)
                rank[r] = (x[u][r] != x[u][r]) ? n_thr[u] : b[u][r].lo;  // NaN is right of every threshold
            const int reg0 = vfirst[f0 + u];
            for (int s = 0, first = 0; first < n_thr[u]; ++s, first += RANK_SEG) {
                const int len = n_thr[u] - first < RANK_SEG ? n_thr[u] - first : RANK_SEG;
                uint32_t packed = 0;
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    int rv = rank[r] - first;
                    rv = rv < 0 ? 0 : (rv > len ? len : rv);
                    packed |= static_cast<uint32_t>(rank_code_bits(rv)) << (16 * r);
                }
                rk[(reg0 + s - reg_begin) * TILE + lane] = packed;
            }
        }
    }
}

// All features, all rank registers.
template <int NWAVES, int U = 2, bool STREAM_X = false>
__device__ __forceinline__ void rank_rows(uint32_t *rk, const DevModel &m, const float *__restrict__ X,
                                          int64_t row0, int64_t n_rows, int wave, int lane)
{
    rank_rows<NWAVES, U, STREAM_X>(rk, m, X, row0, n_rows, wave, lane, 0, m.n_features, 0, m.rank_regs);
}


// ---------------------------------------------------------------------------------------
// The comparison through the vector-register index mode, shared by the kernels that keep their
// rank registers in VGPRs.
// ---------------------------------------------------------------------------------------
typedef uint32_t v32u __attribute__((ext_vector_type(32)));


#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) uint32_t *ProgPtr;
typedef const __attribute__((address_space(4))) TreeMeta *MetaPtr;
#else
typedef const uint32_t *ProgPtr;  // host pass: the kernel body is only parsed
typedef const TreeMeta *MetaPtr;
#endif

// One entry of the compact split program is one scalar register: -4 code(j') in the high half,
// the rank register's index in the low byte.  s_set_gpr_idx_* reads only the low byte; the
// packed multiply-add reads the high half for both rows (op_sel / op_sel_hi of the addend) and
// the inline constant's low half for both (op_sel_hi 0: a packed inline constant fills only it).
// The index mode lives in M0.  M0 is a register the compiler reserves: it never keeps a value of
// its own in it across an inline-assembly statement (it sets M0 immediately before each use it
// generates, and rejects M0 on a clobber list as having no effect), so the statements below may
// write it freely.
struct Entry8 {
    uint32_t e[8];
};

template <int N>
struct Batch {
    Entry8 q[N / 8];
};

template <int N>
__device__ __forceinline__ Batch<N> load_batch(ProgPtr p)
{
    Batch<N> b;
#pragma unroll
    for (int j = 0; j < N; ++j) b.q[j / 8].e[j % 8] = p[j];
    return b;
}


}  // namespace forest_impl
