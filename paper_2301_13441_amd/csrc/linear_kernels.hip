// Linear models on gfx950: raw = X . W + b, transform, label (Section 3.3, Table 4; the label
// comes from the values before the transform, Section 4.3.3).
//
// The path is bound by reading X once from HBM (4 F bytes per row against 2 F K flops), so the
// kernel is a streaming one.  A wavefront owns 64 consecutive rows and walks the features in
// chunks of 32: the 64 x 32 chunk is read coalesced (a half-wave covers 128 contiguous bytes
// of a row), parked in the wave's own LDS tile with an odd row stride, and then every lane
// takes its row out of the tile and accumulates its K outputs in float64 against weights that
// are wave-uniform (scalar loads).  No barriers: the four waves of a workgroup never share
// data, and LDS operations of one wave complete in order.  Products of float32 values are
// exact in float64 and vector float64 FMA runs at full rate on this chip, so the float64
// accumulation costs no bandwidth.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/linear.h"
#include "linear_device.hpp"

namespace linear_impl {
namespace {

// The weights are wave-uniform and never written: reading them through the constant address
// space makes them scalar loads whatever else the kernel does to memory.
#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) double *WeightPtr;
#else
typedef const double *WeightPtr;  // host pass: the kernel body is only parsed
#endif

constexpr int LANES = 64;
constexpr int LWAVES = 4;
constexpr int CHUNK = 32;          // features per pass
constexpr int STRIDE = CHUNK + 4;  // row pitch of the LDS tile in floats: 16-byte aligned rows, and the
                                   // 8 lanes of a 128-bit read phase fall into 8 different bank groups

// Label, transform and store of one row whose K raw values (bias included) are acc[0..K).
// A score to its place.  With one output per row the lanes of a wave write one contiguous piece
// and nothing reads it again here: a non-temporal store (l2: 5 % faster).  With several outputs
// a lane's values are a short run of its own, and stores that skip the cache would each become
// a partial write to memory (l3: twice as slow), so those go the ordinary way.
template <int KP>
__device__ __forceinline__ void store_score(float v, float *p)
{
    if (KP == 1) __builtin_nontemporal_store(v, p);
    else *p = v;
}
template <int KP>
__device__ __forceinline__ void finish_linear_row(const LinDev &m, double (&acc)[KP], int64_t row, float *scores,
                                                  int32_t *labels)
{
    const int K = m.n_outputs;
    double best = acc[0];
    int best_k = 0;
#pragma unroll
    for (int k = 1; k < KP; ++k)
        if (k < K && acc[k] > best) {
            best = acc[k];
            best_k = k;
        }
    if (labels) {
        int lab = best_k;
        if (K == 1) lab = (m.transform == LINEAR_TRANSFORM_SIGMOID) ? (best > 0.0) : (best > 0.5);
        if (KP == 1) __builtin_nontemporal_store(lab, &labels[row]);  // as the scores below
        else labels[row] = lab;
    }
    if (!scores) return;
    float *dst = scores + row * K;
    if (m.transform == LINEAR_TRANSFORM_SOFTMAX) {
        double z = 0.0;
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) {
                acc[k] = exp(acc[k] - best);
                z += acc[k];
            }
        const double inv = 1.0 / z;  // one division per row; the product differs from the quotient by
                                     // at most an ulp of float64, far below the float32 rounding
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) store_score<KP>(static_cast<float>(acc[k] * inv), &dst[k]);
    } else if (m.transform == LINEAR_TRANSFORM_SIGMOID) {
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) store_score<KP>(static_cast<float>(1.0 / (1.0 + exp(-acc[k]))), &dst[k]);
    } else {
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) store_score<KP>(static_cast<float>(acc[k]), &dst[k]);
    }
}

// The lane's share of a 64 x 32 chunk, as V-float pieces: piece i is columns [V * (lane % (32 / V)),
// +V) of row i * (64 * V / 32) + lane / (32 / V), so that 32 / V consecutive lanes read 128
// contiguous bytes of one row.
template <int V>
struct Piece {
    float v[V];
};

template <int V>
__device__ __forceinline__ void load_chunk(Piece<V> (&pre)[CHUNK / V], const float *__restrict__ src, int F, int c0,
                                           int fc, int rows_here, int lane)
{
    constexpr int LPR = CHUNK / V;       // lanes per row
    constexpr int RPI = LANES / LPR;     // rows per instruction
    const int c = (lane % LPR) * V;
#pragma unroll
    for (int i = 0; i < CHUNK / V; ++i) {
        // V divides F and the chunk start, so a piece is inside the matrix or outside as a whole;
        // a piece outside reads the tile's first floats instead (always there) and becomes zero:
        // no branch, every load of the chunk is issued back to back
        const int r = i * RPI + lane / LPR;
        const bool in = r < rows_here && c < fc;
        const float *q = in ? src + static_cast<int64_t>(r) * F + c0 + c : src;
        if (V == 4) {
            const float4 t = *reinterpret_cast<const float4 *>(q);
            pre[i].v[0] = in ? t.x : 0.0f, pre[i].v[1 % V] = in ? t.y : 0.0f;
            pre[i].v[2 % V] = in ? t.z : 0.0f, pre[i].v[3 % V] = in ? t.w : 0.0f;
        } else if (V == 2) {
            const float2 t = *reinterpret_cast<const float2 *>(q);
            pre[i].v[0] = in ? t.x : 0.0f, pre[i].v[1 % V] = in ? t.y : 0.0f;
        } else {
            const float t = *q;
            pre[i].v[0] = in ? t : 0.0f;
        }
    }
}

// The same pieces when the tile has all 64 rows and the chunk all 32 columns (every tile and chunk
// but the last ones): nothing to test, and nothing is done to the values once they are requested,
// so the loads stay in flight until the chunk is parked.  `chunk` is the tile's first row at the
// chunk's first column (wave-uniform), `lane_bytes` the lane's place in piece 0.
template <int V>
__device__ __forceinline__ void load_chunk_full(Piece<V> (&pre)[CHUNK / V], const float *__restrict__ chunk, int F,
                                                uint32_t lane_bytes)
{
    constexpr int RPI = LANES / (CHUNK / V);
#pragma unroll
    for (int i = 0; i < CHUNK / V; ++i) {
        const char *q = reinterpret_cast<const char *>(chunk + static_cast<int64_t>(i) * RPI * F) + lane_bytes;
        if (V == 4) {
            typedef float F4 __attribute__((ext_vector_type(4)));
            const F4 t = __builtin_nontemporal_load(reinterpret_cast<const F4 *>(q));  // read once, not to be kept
            pre[i].v[0] = t.x, pre[i].v[1 % V] = t.y, pre[i].v[2 % V] = t.z, pre[i].v[3 % V] = t.w;
        } else if (V == 2) {
            const float2 t = *reinterpret_cast<const float2 *>(q);
            pre[i].v[0] = t.x, pre[i].v[1 % V] = t.y;
        } else {
            pre[i].v[0] = *reinterpret_cast<const float *>(q);
        }
    }
}

template <int V>
__device__ __forceinline__ void park_chunk(float *xs, const Piece<V> (&pre)[CHUNK / V], int lane)
{
    constexpr int LPR = CHUNK / V;
    constexpr int RPI = LANES / LPR;
    const int c = (lane % LPR) * V;
#pragma unroll
    for (int i = 0; i < CHUNK / V; ++i) {
        float *d = xs + (i * RPI + lane / LPR) * STRIDE + c;
        if (V == 4) *reinterpret_cast<float4 *>(d) = make_float4(pre[i].v[0], pre[i].v[1 % V], pre[i].v[2 % V], pre[i].v[3 % V]);
        else if (V == 2) *reinterpret_cast<float2 *>(d) = make_float2(pre[i].v[0], pre[i].v[1 % V]);
        else *d = pre[i].v[0];
    }
}

// V: floats per global load (4 when rows are 16-byte aligned, i.e. F % 4 == 0; else 2 or 1).
template <int KP, int V>
__global__ __launch_bounds__(LANES *LWAVES) void linear_kernel(LinDev m, const float *__restrict__ X,
                                                                int64_t n_rows, float *scores, int32_t *labels)
{
    __shared__ __align__(16) float tile[LWAVES][LANES * STRIDE];
    const int lane = threadIdx.x & (LANES - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float *xs = tile[wave];
    const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * LWAVES + wave) * LANES;
    if (row0 >= n_rows) return;  // wave-uniform
    const int F = m.n_features;
    const int64_t left = n_rows - row0;
    const int rows_here = left < LANES ? static_cast<int>(left) : LANES;
    const float *__restrict__ src = X + row0 * F;

    double acc[KP];
#pragma unroll
    for (int k = 0; k < KP; ++k) acc[k] = m.bias[k];

    // Chunks that are whole (all 64 rows, all 32 columns) go through a loop of fixed shape: two
    // chunks are on their way from HBM, held in registers, while the current one is used, and every
    // step requests eight loads -- past the last whole chunk they all read the tile's first floats,
    // one cache line, and are dropped -- so the number of loads between a request and its use is
    // known and a wave waits only for the chunk it is about to park.  What is left (the last
    // columns of a matrix whose width is not a multiple of 32; every chunk of the last tile) goes
    // one chunk at a time through the loads that test and mask.
    Piece<V> pre0[CHUNK / V], pre1[CHUNK / V];
    const int n_whole = rows_here == LANES ? F / CHUNK : 0;  // wave-uniform
    const uint32_t lane_bytes =
        static_cast<uint32_t>(sizeof(float)) * (static_cast<uint32_t>(lane / (CHUNK / V)) * static_cast<uint32_t>(F) + (lane % (CHUNK / V)) * V);
    auto fetch = [&](Piece<V> (&pre)[CHUNK / V], int chunk) {
        const bool there = chunk < n_whole;
        load_chunk_full<V>(pre, there ? src + chunk * CHUNK : src, there ? F : 0, there ? lane_bytes : 0u);
    };
    // The feature loop runs through all chunks as one stream of weights.
    WeightPtr w = (WeightPtr)m.weight;
    auto use = [&]() {
        // the tile holds zeros past the last feature and the weight matrix has zero rows there,
        // so every chunk runs all 32 columns without a test
        const float4 *row = reinterpret_cast<const float4 *>(xs + lane * STRIDE);
#pragma unroll 2
        for (int c = 0; c < CHUNK; c += 4) {
            const float4 t = row[c >> 2];
            const float x4[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double x = static_cast<double>(x4[j]);
#pragma unroll
                for (int k = 0; k < KP; ++k) acc[k] = __builtin_fma(x, w[j * KP + k], acc[k]);
            }
            w += 4 * KP;
        }
    };
    int chunk = 0;
    if (n_whole > 0) {
        fetch(pre0, 0);
        fetch(pre1, 1);
        for (; chunk + 2 <= n_whole; chunk += 2) {
            park_chunk<V>(xs, pre0, lane);
            fetch(pre0, chunk + 2);
            use();
            park_chunk<V>(xs, pre1, lane);
            fetch(pre1, chunk + 3);
            use();
        }
        if (chunk < n_whole) {
            park_chunk<V>(xs, pre0, lane);
            use();
            ++chunk;
        }
    }
    for (int c0 = chunk * CHUNK; c0 < F; c0 += CHUNK) {
        load_chunk<V>(pre0, src, F, c0, F - c0 < CHUNK ? F - c0 : CHUNK, rows_here, lane);
        park_chunk<V>(xs, pre0, lane);
        use();
    }

    if (lane < rows_here) finish_linear_row<KP>(m, acc, row0 + lane, scores, labels);
}

// Narrow matrices (a 64-row tile of whole rows fits the wave's share of LDS): the tile is one
// contiguous piece of X, copied to LDS as it lies in memory by loads that write LDS directly
// (global_load_lds, 16 bytes per lane, no register staging): every byte of X is requested once,
// in 1 KB pieces, and all of a tile's loads are in flight at once.  Rows whose size is not a
// multiple of the 128-byte line would otherwise be fetched twice by the chunked kernel, once for
// each chunk a line straddles.
constexpr int ROWS_WAVES = 2;
constexpr int ROWS_MAX_FEATURES = 96;

template <int KP>
__global__ __launch_bounds__(LANES *ROWS_WAVES) void linear_rows_kernel(LinDev m, const float *__restrict__ X,
                                                                         int64_t n_rows, float *scores,
                                                                         int32_t *labels)
{
    extern __shared__ __align__(16) float rows_tile[];  // [ROWS_WAVES][64 * F]
    const int lane = threadIdx.x & (LANES - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int F = m.n_features;
    float *xs = rows_tile + wave * LANES * F;
    const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * ROWS_WAVES + wave) * LANES;
    if (row0 >= n_rows) return;  // wave-uniform
    const int64_t left = n_rows - row0;
    const int rows_here = left < LANES ? static_cast<int>(left) : LANES;
    const float *__restrict__ src = X + row0 * F;  // 16-byte aligned: 64 F floats per tile
    const int n = rows_here * F, n4 = n >> 2;
#if defined(__HIP_DEVICE_COMPILE__)
    typedef __attribute__((address_space(1))) const void *GlobalPtr;
    typedef __attribute__((address_space(3))) void *LdsPtr;
    for (int i = 0; i * LANES < n4; ++i) {
        if (i * LANES + lane < n4)  // the LDS address is the wave-uniform base plus 16 bytes per lane
            __builtin_amdgcn_global_load_lds((GlobalPtr)(src + (i * LANES + lane) * 4), (LdsPtr)(xs + i * LANES * 4), 16, 0, 2 /* non-temporal: X is read once, not to be kept (l4 12 % faster, l2 8 %) */);
    }
#endif
    for (int e = n4 * 4 + lane; e < n; e += LANES) xs[e] = src[e];  // at most three floats of a partial tile
    double acc[KP];
#pragma unroll
    for (int k = 0; k < KP; ++k) acc[k] = ((WeightPtr)m.bias)[k];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const float *row = xs + (lane < rows_here ? lane : 0) * F;
    WeightPtr w = (WeightPtr)m.weight;
#pragma unroll 8
    for (int f = 0; f < F; ++f) {
        const double x = static_cast<double>(row[f]);
#pragma unroll
        for (int k = 0; k < KP; ++k) acc[k] = __builtin_fma(x, w[f * KP + k], acc[k]);
    }
    if (lane < rows_here) finish_linear_row<KP>(m, acc, row0 + lane, scores, labels);
}

using LinearFn = void (*)(LinDev, const float *, int64_t, float *, int32_t *);

template <int V>
LinearFn pick_k(int kp)
{
    switch (kp) {
        case 1: return linear_kernel<1, V>;
        case 2: return linear_kernel<2, V>;
        case 3: return linear_kernel<3, V>;
        case 4: return linear_kernel<4, V>;
        case 5: return linear_kernel<5, V>;
        case 6: return linear_kernel<6, V>;
        case 8: return linear_kernel<8, V>;
        case 10: return linear_kernel<10, V>;
        case 12: return linear_kernel<12, V>;
        case 16: return linear_kernel<16, V>;
        case 24: return linear_kernel<24, V>;
        case 32: return linear_kernel<32, V>;
        default: return nullptr;
    }
}

LinearFn pick_rows(int kp)
{
    switch (kp) {
        case 1: return linear_rows_kernel<1>;
        case 2: return linear_rows_kernel<2>;
        case 3: return linear_rows_kernel<3>;
        case 4: return linear_rows_kernel<4>;
        case 5: return linear_rows_kernel<5>;
        case 6: return linear_rows_kernel<6>;
        case 8: return linear_rows_kernel<8>;
        case 10: return linear_rows_kernel<10>;
        case 12: return linear_rows_kernel<12>;
        case 16: return linear_rows_kernel<16>;
        case 24: return linear_rows_kernel<24>;
        case 32: return linear_rows_kernel<32>;
        default: return nullptr;
    }
}

// Widest load that every row start and every chunk start is aligned for.
LinearFn pick(int kp, int n_features, const float *X)
{
    const bool a16 = (reinterpret_cast<uintptr_t>(X) & 15) == 0, a8 = (reinterpret_cast<uintptr_t>(X) & 7) == 0;
    if (n_features % 4 == 0 && a16) return pick_k<4>(kp);
    if (n_features % 2 == 0 && a8) return pick_k<2>(kp);
    return pick_k<1>(kp);
}

}  // namespace

int padded_outputs(int n_outputs)
{
    static const int sizes[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32};
    for (int s : sizes)
        if (s >= n_outputs) return s;
    return 0;
}

hipError_t launch_linear(const LinDev &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                         hipStream_t stream)
{
    if (n_rows <= 0) return hipSuccess;
    if (m.n_features <= ROWS_MAX_FEATURES && (reinterpret_cast<uintptr_t>(X) & 15) == 0) {
        LinearFn fn = pick_rows(m.kp);
        if (!fn) return hipErrorInvalidValue;
        const int64_t rows_per_block = LANES * ROWS_WAVES;
        const int64_t n_blocks = (n_rows + rows_per_block - 1) / rows_per_block;
        if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        const size_t lds = sizeof(float) * ROWS_WAVES * LANES * m.n_features;
        hipLaunchKernelGGL(fn, dim3(static_cast<unsigned>(n_blocks)), dim3(LANES * ROWS_WAVES), lds, stream, m, X,
                           n_rows, scores, labels);
        return hipGetLastError();
    }
    LinearFn fn = pick(m.kp, m.n_features, X);
    if (!fn) return hipErrorInvalidValue;
    const int64_t n_blocks = (n_rows + LANES * LWAVES - 1) / (LANES * LWAVES);
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, dim3(static_cast<unsigned>(n_blocks)), dim3(LANES * LWAVES), 0, stream, m, X, n_rows,
                       scores, labels);
    return hipGetLastError();
}

}  // namespace linear_impl
