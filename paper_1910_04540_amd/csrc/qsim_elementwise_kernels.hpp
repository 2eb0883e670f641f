// Elementwise kernels of libqsim: custom floating point and fixed point.
#pragma once

#include "qsim_kernel_common.hpp"

namespace qsim {

// ---------------------------------------------------------------------------------------------
// Elementwise quantizers with the format resolved at compile time (aligned arrays).
// ---------------------------------------------------------------------------------------------
struct FixedOp {
    GridPlan plan;
    template <int MODE>
    __device__ __forceinline__ uint32_t apply(uint32_t bits, uint32_t r) const
    {
        return quantize_to_grid<MODE>(bits, plan, r);
    }
};

template <bool DENORMAL_INPUTS>
struct FloatShiftOp {
    FloatPlan plan;
    template <int MODE>
    __device__ __forceinline__ uint32_t apply(uint32_t bits, uint32_t r) const
    {
        return quantize_float_shift<MODE, DENORMAL_INPUTS>(bits, plan, r);
    }
};

struct FloatGeneralOp {
    FloatPlan plan;
    template <int MODE>
    __device__ __forceinline__ uint32_t apply(uint32_t bits, uint32_t r) const
    {
        return quantize_float_general<MODE>(bits, plan, r);
    }
};

// One wavefront per workgroup: measured a little faster than 256 threads for pure streaming
// (6.65 against 6.52 TB/s for a plain copy), and these kernels share nothing inside a workgroup.
constexpr int kStreamThreads = 64;

template <class Op, int MODE, int UNROLL>
__global__ __launch_bounds__(kStreamThreads) void elementwise_kernel(const uint32_t* in, uint32_t* out, uint64_t n,
                                                                     uint64_t groups, Op op, RngKey key)
{
    const uint64_t base = linear_block() * (kStreamThreads * UNROLL) + threadIdx.x;
    uint4 v[UNROLL];
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint64_t j = base + (uint64_t)k * kStreamThreads;
        if (j < groups) v[k] = load_group<true>(in, j, n);
    }
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint64_t j = base + (uint64_t)k * kStreamThreads;
        if (j < groups) {
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (MODE == QSIM_STOCHASTIC) r = random_words(j, key, 0u);
            uint4 o;
            o.x = op.template apply<MODE>(v[k].x, r.w[0]);
            o.y = op.template apply<MODE>(v[k].y, r.w[1]);
            o.z = op.template apply<MODE>(v[k].z, r.w[2]);
            o.w = op.template apply<MODE>(v[k].w, r.w[3]);
            store_group<true>(out, j, n, o);
        }
    }
}

// Float or fixed format chosen at run time, dword accesses: the path for unaligned arrays.
__global__ __launch_bounds__(kThreads) void elementwise_rt_kernel(const uint32_t* in, uint32_t* out, uint64_t n,
                                                                  uint64_t groups, FormatPlan f, RngKey key)
{
    const uint64_t j = linear_block() * kThreads + threadIdx.x;
    if (j >= groups) return;
    const uint4 v = load_group<false>(in, j, n);
    Words4 r = {{0u, 0u, 0u, 0u}};
    if (f.mode == QSIM_STOCHASTIC) r = random_words(j, key, 0u);
    store_group<false>(out, j, n, quantize_group_rt(f, f.grid, v, r));
}

}  // namespace qsim
