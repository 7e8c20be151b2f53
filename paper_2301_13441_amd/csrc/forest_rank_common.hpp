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
// (register v of the group: first entry in bit 7), i = 1 the row-b bytes; a second matrix
// weighs by 2^(15 - v).  Two chained MFMAs on top of a 2^23 addend therefore leave the 16
// outcome bits of two groups in the low mantissa bits of D[..][0] and D[..][1]: exact, every
// product and partial sum being an integer below 2^24.  The matrix core runs beside the
// vector ALU, so collecting a group costs the vector ALU the MFMA's issue instead of the eight
// instructions of a packed fused-multiply-add tree.
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

struct BitCollector {
    v8i a[2];  // weights 2^(7 - v) and 2^(15 - v)
    v4f bias;

    __device__ __forceinline__ void init(int lane)
    {
        const int m = lane & 15, q = lane >> 4;
        const bool mine = (m >> 2) == q && (m & 3) < 2;
        const int shift = (m & 3) == 0 ? 8 : 24;  // byte 1 = row a, byte 3 = row b
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                const uint32_t bf8 = static_cast<uint32_t>(15 + 8 * j + 7 - v) << 2;  // 2^(8j + 7 - v)
                a[j][v] = mine ? static_cast<int>(bf8 << shift) : 0;
            }
        bias = v4f{8388608.0f, 8388608.0f, 8388608.0f, 8388608.0f};
        // keep the addend in registers instead of rebuilding it before every chain
        asm volatile("" : "+v"(bias));
    }
    // the same with the eight outcome registers already in one tuple (weights 2^(7 - v))
    __device__ __forceinline__ v4f collect_b(const v8i &b, v4f c) const
    {
#if defined(__HIP_DEVICE_COMPILE__)
        c = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[0], b, c, 1, 1, 0, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#endif
        return c;
    }
    template <int J>
    __device__ __forceinline__ v4f collect(const uint32_t (&d)[8], v4f c) const
    {
#if defined(__HIP_DEVICE_COMPILE__)
        const v8i b = {static_cast<int>(d[0]), static_cast<int>(d[1]), static_cast<int>(d[2]), static_cast<int>(d[3]),
                       static_cast<int>(d[4]), static_cast<int>(d[5]), static_cast<int>(d[6]), static_cast<int>(d[7])};
        c = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a[J], b, c, 1, 1, 0, 0, 0, 0);  // A, B: bf8, unscaled
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
                                              int n_valid)
{
    const int F = m.n_features;
    const int n_threads = NWAVES * TILE;
    for (int i = threadIdx.x; i < m.rank_regs * TILE; i += n_threads) rk[i] = 0;
    __syncthreads();
    uint16_t *rk16 = reinterpret_cast<uint16_t *>(rk);
    for (int w = threadIdx.x; w < n_valid * F; w += n_threads) {
        const int r = w / F, f = w - r * F;
        store_rank(rk16, m, f, r, rank_of(m, f, Xt[w]));
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

// Ranks of rows [row0, row0 + 128) for every feature with thresholds, written as packed f16
// pairs into rk[reg * 64 + lane] (low half: row `lane` of the tile, high half: row lane + 64).
// The features are dealt to the waves; inside a wave every lane looks up the same feature for
// its own two rows, U features at a time (2 U lookups in flight per lane), so the feature's
// constants are read with scalar loads.  A lookup is a bucket (a subtraction, a multiplication,
// a conversion), the bucket's bracket from the start table, the check of the bracket against
// the two thresholds next to it, and the rank inside the bracket (a count over 8 thresholds, or
// a binary search).
template <int NWAVES, int U = 2, bool STREAM_X = false>
__device__ __forceinline__ void rank_rows(uint32_t *rk, const DevModel &m, const float *__restrict__ X,
                                          int64_t row0, int64_t n_rows, int wave, int lane)
{
    const int F = m.n_features;
    const int64_t left = n_rows - row0;
    if (left * 4 <= RROWS) {  // workgroup-uniform
        rank_rows_few<NWAVES>(rk, m, X + row0 * F, static_cast<int>(left));
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
    for (int f0 = wave * U; f0 < F; f0 += NWAVES * U) {
        float x[U][2];
        RankBracket b[U][2];
        int tb[U], n_thr[U];
        FeatBucket fb[U];
        // all feature values first, then all bucket reads: the loads of one kind go out together
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int f = f0 + u < F ? f0 + u : F - 1;  // wave-uniform; the duplicate is not stored
            tb[u] = thr_base[f];
            n_thr[u] = thr_base[f + 1] - tb[u];
            fb[u].lo = buckets[f].lo;
            fb[u].scale = buckets[f].scale;
            fb[u].n_buckets = buckets[f].n_buckets;
            fb[u].start_base = buckets[f].start_base;
            if (f0 + U > F) {
#pragma unroll
                for (int r = 0; r < 2; ++r)
                    x[u][r] = xrow[r][f];  // a row past the batch reads the tile's first row; its rank is not used
            }
        }
        if (f0 + U <= F) {  // wave-uniform: the U neighbouring features of a row in one load
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
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int r = 0; r < 2; ++r) b[u][r] = bucket_bracket(fb[u], m.bucket_start, x[u][r]);
        // Check of the bracket and the rank inside it.  A feature with 8 thresholds or more
        // (wave-uniform) reads, besides the two neighbours of the check, the 8 thresholds from
        // start = min(lo, n - 8) on: if the bracket holds, every threshold below lo is < x and
        // none from hi on is, so rank = start + #{i < 8 : thr[start + i] < x} whenever hi <= start + 8
        // -- no search.  What is left open (a bracket that does not hold, or a wider one, or a
        // feature with fewer thresholds) goes through the binary search below.
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float *thr = m.thr_sorted + tb[u];
            const int n = n_thr[u];
            if (n >= 8) {
                float tl[2], th[2];
                FloatRun<8> w[2];
                int start[2];
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const RankBracket c = b[u][r];
                    start[r] = c.lo < n - 8 ? c.lo : n - 8;
                    tl[r] = load_at<float>(thr, static_cast<uint32_t>(c.lo > 0 ? c.lo - 1 : 0) << 2);
                    th[r] = load_at<float>(thr, static_cast<uint32_t>(c.hi < n - 1 ? c.hi : n - 1) << 2);
                    w[r] = load_at<FloatRun<8>>(thr, static_cast<uint32_t>(start[r]) << 2);
                }
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    const RankBracket c = b[u][r];
                    const float xv = x[u][r];
                    const bool ok = ((c.lo == 0) | (tl[r] < xv)) & ((c.hi == n) | !(th[r] < xv));
                    int rank = start[r];
#pragma unroll
                    for (int i = 0; i < 8; ++i) rank += (w[r].v[i] < xv) ? 1 : 0;
                    const bool closed = ok & (c.hi <= start[r] + 8);
                    b[u][r].lo = closed ? rank : (ok ? c.lo : 0);
                    b[u][r].hi = closed ? rank : (ok ? c.hi : n);
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
            if (f0 + u >= F) continue;
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
                rk[(reg0 + s) * TILE + lane] = packed;
            }
        }
    }
}

}  // namespace forest_impl
