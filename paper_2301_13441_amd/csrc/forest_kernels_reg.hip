// Register-resident kernels for full trees (gfx950).
//
// The dense evaluation of Fig. 2 costs one comparison per (row, internal node); everything
// else must cost next to nothing.  Here the wave keeps the features of its rows in vector
// registers (lane = row, register = feature) and selects the register with the hardware's
// VGPR index mode (s_set_gpr_idx_on: M0 holds the wave-uniform feature index), so step (1)
// "matmul(X, W1)" costs no instruction of its own.  Per entry of the split program and per
// row slot the wave issues
//     v_cmp_nle_f32   mask, x[feature], threshold      -- step (2), greater(., W2), NaN -> right
//     v_addc_co_u32   word, word, word, mask           -- word = 2 * word + outcome
// i.e. two vector instructions per (row, node).  Two row slots per lane (R = 2) share one
// index-mode switch, which keeps the scalar unit off the critical path and separates each
// v_cmp from the v_addc that consumes its mask by the two independent instructions gfx950
// requires between a VALU write of an SGPR and a VALU read of it.
//
// The feature vectors are pinned to fixed registers (v64 and up) because the index mode
// addresses registers relative to a base named in the instruction text.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "forest_device.hpp"
#include "forest_kernel_common.hpp"

namespace forest_impl {
namespace {

typedef float v32f __attribute__((ext_vector_type(32)));

// step(): apply one split-program entry to every row slot of the lane.
template <int NV, int R>
struct RegStep;

template <>
struct RegStep<1, 2> {
    static __device__ __forceinline__ void step(uint32_t (&b)[2], int f, float t, const v32f (&x)[2][1])
    {
        uint64_t m1;
        asm volatile(
            "s_set_gpr_idx_on %[f], 0x1\n\t"
            "v_cmp_nle_f32_e64 vcc, v64, %[t]\n\t"
            "v_cmp_nle_f32_e64 %[m1], v96, %[t]\n\t"
            "s_set_gpr_idx_off\n\t"
            "v_addc_co_u32_e32 %[b0], vcc, %[b0], %[b0], vcc\n\t"
            "v_addc_co_u32_e64 %[b1], vcc, %[b1], %[b1], %[m1]"
            : [b0] "+v"(b[0]), [b1] "+v"(b[1]), [m1] "=&s"(m1)
            : [f] "s"(f), [t] "s"(t), "{v[64:95]}"(x[0][0]), "{v[96:127]}"(x[1][0])
            : "vcc");
    }
};

template <>
struct RegStep<2, 2> {
    static __device__ __forceinline__ void step(uint32_t (&b)[2], int f, float t, const v32f (&x)[2][2])
    {
        uint64_t m1;
        asm volatile(
            "s_set_gpr_idx_on %[f], 0x1\n\t"
            "v_cmp_nle_f32_e64 vcc, v64, %[t]\n\t"
            "v_cmp_nle_f32_e64 %[m1], v128, %[t]\n\t"
            "s_set_gpr_idx_off\n\t"
            "v_addc_co_u32_e32 %[b0], vcc, %[b0], %[b0], vcc\n\t"
            "v_addc_co_u32_e64 %[b1], vcc, %[b1], %[b1], %[m1]"
            : [b0] "+v"(b[0]), [b1] "+v"(b[1]), [m1] "=&s"(m1)
            : [f] "s"(f), [t] "s"(t), "{v[64:95]}"(x[0][0]), "{v[96:127]}"(x[0][1]),
              "{v[128:159]}"(x[1][0]), "{v[160:191]}"(x[1][1])
            : "vcc");
    }
};

template <>
struct RegStep<4, 1> {
    static __device__ __forceinline__ void step(uint32_t (&b)[1], int f, float t, const v32f (&x)[1][4])
    {
        asm volatile(
            "s_set_gpr_idx_on %[f], 0x1\n\t"
            "v_cmp_nle_f32_e64 vcc, v64, %[t]\n\t"
            "s_set_gpr_idx_off\n\t"
            "s_nop 0\n\t"
            "v_addc_co_u32_e32 %[b0], vcc, %[b0], %[b0], vcc"
            : [b0] "+v"(b[0])
            : [f] "s"(f), [t] "s"(t), "{v[64:95]}"(x[0][0]), "{v[96:127]}"(x[0][1]),
              "{v[128:159]}"(x[0][2]), "{v[160:191]}"(x[0][3])
            : "vcc");
    }
};

template <int N>
struct Batch {
    SplitEntry e[N];
};

// The packed model is immutable while a kernel runs: reading it through the constant address
// space makes every wave-uniform read a scalar load, whatever else the kernel stores.
#if defined(__HIP_DEVICE_COMPILE__)
typedef const __attribute__((address_space(4))) SplitEntry *ProgPtr;
#else
typedef const SplitEntry *ProgPtr;  // host pass: the kernel body is only parsed
#endif

template <int N>
__device__ __forceinline__ Batch<N> load_batch(ProgPtr p)
{
    Batch<N> b;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        b.e[j].feature_slot = p[j].feature_slot;
        b.e[j].threshold = p[j].threshold;
    }
    return b;
}

template <int D, int NV, int R>
__global__ __launch_bounds__(BLOCK) void forest_reg_kernel(DevModel m, const float *__restrict__ X,
                                                           int64_t n_rows, float *scores,
                                                           int32_t *labels, int32_t *leaf_out)
{
    constexpr int ROWS = TILE * R;
    constexpr int FCAP = 32 * NV;
    extern __shared__ __align__(16) char smem[];
    double *acc = reinterpret_cast<double *>(smem);                        // [WAVES][K][ROWS]
    float *xs = reinterpret_cast<float *>(smem + sizeof(double) * WAVES * m.n_outputs * ROWS);  // [FCAP][ROWS]

    const int lane = threadIdx.x & (TILE - 1);
    const int wave = uniform(threadIdx.x >> 6);
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * ROWS;
    const int F = m.n_features;

    stage_x_tile(xs, X, row0, n_rows, F, ROWS);
    for (int e = F * ROWS + threadIdx.x; e < FCAP * ROWS; e += BLOCK) xs[e] = 0.0f;
    __syncthreads();

    v32f x[R][NV];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int i = 0; i < 32; ++i) x[r][v][i] = xs[(v * 32 + i) * ROWS + r * TILE + lane];

    const bool LEAVES = leaf_out != nullptr;  // wave-uniform: debug output instead of scores
    Accumulator<R> accu;
    accu.init(acc, wave, lane, m);

    constexpr int N_POS = 1 << D;
    constexpr int BLK = N_POS < 32 ? N_POS : 32;   // entries per outcome word
    constexpr int NW = N_POS / BLK;                // outcome words per tree
    constexpr int NB = BLK < 16 ? BLK : 16;        // entries per scalar load batch
    const int T = m.n_trees;
    int t_begin, t_end;
    tree_range(m, wave, WAVES, t_begin, t_end);

    // The wave's trees are one contiguous stream of entries; the batch after the last one
    // read here is padding the host appended to the program.
    ProgPtr p = (ProgPtr)(m.prog + (static_cast<size_t>(t_begin) << D));
    Batch<NB> cur = load_batch<NB>(p);
    for (int t = t_begin; t < t_end; ++t) {
        uint32_t word[R][NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            uint32_t b[R];
#pragma unroll
            for (int r = 0; r < R; ++r) b[r] = 0;
#pragma unroll
            for (int h = 0; h < BLK / NB; ++h) {
                // first entry, then issue the next batch's loads, then the rest: the loads
                // are in flight while this batch is evaluated
                RegStep<NV, R>::step(b, cur.e[0].feature_slot, cur.e[0].threshold, x);
                p += NB;
                const Batch<NB> nxt = load_batch<NB>(p);
#pragma unroll
                for (int j = 1; j < NB; ++j)
                    RegStep<NV, R>::step(b, cur.e[j].feature_slot, cur.e[j].threshold, x);
                cur = nxt;
            }
#pragma unroll
            for (int r = 0; r < R; ++r) word[r][w] = b[r];
        }
        const TreeMeta tm = m.tree[t];
        if (!LEAVES) accu.begin_tree(tm.column);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int leaf = (t << D) + static_cast<int>(heap_walk<D, NW>(word[r]));
            if (LEAVES) {
                const int64_t row = row0 + r * TILE + lane;
                if (row < n_rows) leaf_out[row * T + tm.caller_tree] = m.leaf_node[leaf];
            } else {
                accu.add(m, r, leaf);
            }
        }
    }
    if (LEAVES) return;
    accu.flush();
    __syncthreads();
    const int li = threadIdx.x;
    if (li < ROWS) finish_row(m, acc, ROWS, li, row0 + li, row0 + li < n_rows, scores, labels);
}

size_t reg_lds_bytes(const DevModel &m)
{
    const int rows = TILE * m.reg_r;
    return sizeof(double) * WAVES * m.n_outputs * rows + sizeof(float) * 32 * m.reg_nv * rows;
}

template <int NV, int R>
KernelFn pick_depth(int d)
{
    switch (d) {
        case 1: return forest_reg_kernel<1, NV, R>;
        case 2: return forest_reg_kernel<2, NV, R>;
        case 3: return forest_reg_kernel<3, NV, R>;
        case 4: return forest_reg_kernel<4, NV, R>;
        case 5: return forest_reg_kernel<5, NV, R>;
        case 6: return forest_reg_kernel<6, NV, R>;
        case 7: return forest_reg_kernel<7, NV, R>;
        case 8: return forest_reg_kernel<8, NV, R>;
        default: return nullptr;
    }
}

KernelFn pick_reg(int nv, int r, int d)
{
    if (nv == 1 && r == 2) return pick_depth<1, 2>(d);
    if (nv == 2 && r == 2) return pick_depth<2, 2>(d);
    if (nv == 4 && r == 1) return pick_depth<4, 1>(d);
    return nullptr;
}

const int kConfigs[3][2] = {{1, 2}, {2, 2}, {4, 1}};

}  // namespace

hipError_t init_reg_kernels(size_t lds_limit)
{
    for (const auto &c : kConfigs)
        for (int d = 1; d <= FULL_MAX_DEPTH; ++d) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(pick_reg(c[0], c[1], d)),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               static_cast<int>(lds_limit));
            if (e != hipSuccess) return e;
        }
    return hipSuccess;
}

hipError_t launch_reg(const DevModel &m, const float *X, int64_t n_rows, float *scores, int32_t *labels,
                      int32_t *leaf_out, hipStream_t stream)
{
    KernelFn fn = pick_reg(m.reg_nv, m.reg_r, m.kind);
    if (!fn) return hipErrorInvalidValue;
    if (m.n_features > 32 * m.reg_nv) return hipErrorInvalidValue;
    const int rows = TILE * m.reg_r;
    const int64_t n_blocks = (n_rows + rows - 1) / rows;
    if (n_blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>(n_blocks), static_cast<unsigned>(m.n_splits));
    hipLaunchKernelGGL(fn, grid, dim3(BLOCK), reg_lds_bytes(m), stream, m, X, n_rows, scores, labels, leaf_out);
    return hipGetLastError();
}

}  // namespace forest_impl
