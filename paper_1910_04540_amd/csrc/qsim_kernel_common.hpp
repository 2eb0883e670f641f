// Kernels of libqsim.  Hand-written HIP for gfx950 (MI355X).
//
// All kernels are streaming: a thread's unit of work is one group of four consecutive elements
// whose first index is a multiple of four, i.e. one dwordx4 load, one Philox4x32-10 block (its
// four words belong to exactly these four elements) and one dwordx4 store.  Loads and stores are
// non-temporal: every byte is touched once.  Arrays that are not 16-byte aligned take the dword
// path of the run-time-format kernels.
#pragma once

#include <hip/hip_runtime.h>
#include "qsim_device.hpp"

namespace qsim {

constexpr int kThreads = 256;

// A dispatch cannot hold 2^32 work-items or more in one dimension, so grids proportional to the
// tensor are folded over x and y (over x and z where y already carries slices): x never exceeds
// kGridX workgroups, and a kernel takes its workgroup number from linear_block().
constexpr unsigned kGridX = 1u << 20;
__device__ __forceinline__ uint64_t linear_block() { return (uint64_t)blockIdx.y * gridDim.x + blockIdx.x; }
__device__ __forceinline__ uint64_t linear_block_xz() { return (uint64_t)blockIdx.z * gridDim.x + blockIdx.x; }

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_at_dword __attribute__((aligned(4)));     // a group at an address that is only dword aligned

__device__ __forceinline__ uint4 to_uint4(u32x4 v) { return make_uint4(v.x, v.y, v.z, v.w); }
__device__ __forceinline__ u32x4 to_u32x4(const uint4& v) { return u32x4{v.x, v.y, v.z, v.w}; }

// ---------------------------------------------------------------------------------------------
// Group access: elements [4*j, 4*j+4) of an array whose valid elements end at `end`.
// VEC: the array is 16-byte aligned.  A whole group is one dwordx4 access either way (global
// memory takes multi-dword accesses at any dword-aligned address; a misaligned one merely touches
// one more cache line per wavefront); only a group cut off by `end` goes element by element.
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__device__ __forceinline__ uint4 load_group(const uint32_t* p, uint64_t j, uint64_t end)
{
    const uint64_t i = j * 4;
    if (i + 4 <= end) {
        if (VEC) return to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p + i)));
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_at_dword*>(p + i));
        return to_uint4(v);
    }
    uint4 v = {0u, 0u, 0u, 0u};
    if (i + 0 < end) v.x = p[i + 0];
    if (i + 1 < end) v.y = p[i + 1];
    if (i + 2 < end) v.z = p[i + 2];
    if (i + 3 < end) v.w = p[i + 3];
    return v;
}

template <bool VEC>
__device__ __forceinline__ void store_group(uint32_t* p, uint64_t j, uint64_t end, const uint4& v)
{
    const uint64_t i = j * 4;
    if (i + 4 <= end) {
        if (VEC) __builtin_nontemporal_store(to_u32x4(v), reinterpret_cast<u32x4*>(p + i));
        else __builtin_nontemporal_store(to_u32x4(v), reinterpret_cast<u32x4_at_dword*>(p + i));
        return;
    }
    if (i + 0 < end) p[i + 0] = v.x;
    if (i + 1 < end) p[i + 1] = v.y;
    if (i + 2 < end) p[i + 2] = v.z;
    if (i + 3 < end) p[i + 3] = v.w;
}


// Workgroup-wide maximum: wave reduction, then one LDS slot per wave.
template <int THREADS = kThreads>
__device__ __forceinline__ uint32_t workgroup_max(uint32_t v, uint32_t* lds /* THREADS / 64 slots */)
{
    const uint32_t w = wave_max(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();                        // protects the slots against the previous use
    if ((threadIdx.x & 63) == 0) lds[wave] = w;
    __syncthreads();
    uint32_t m = lds[0];
#pragma unroll
    for (int k = 1; k < THREADS / 64; ++k) m = m > lds[k] ? m : lds[k];
    return m;
}

template <int MODE>
__device__ __forceinline__ uint4 quantize_group_to_grid(const uint4& v, const GridPlan& p, const Words4& r)
{
    uint4 o;
    o.x = quantize_to_grid<MODE>(v.x, p, r.w[0]);
    o.y = quantize_to_grid<MODE>(v.y, p, r.w[1]);
    o.z = quantize_to_grid<MODE>(v.z, p, r.w[2]);
    o.w = quantize_to_grid<MODE>(v.w, p, r.w[3]);
    return o;
}

// A block's group under the block's plan.  `finite` says that plan_is_finite holds and must be the
// same in every lane of the wavefront: blocks without Inf and NaN, all but a few, take the short
// form of the quantizer.
template <int MODE>
__device__ __forceinline__ uint4 quantize_group_of_block(const uint4& v, const GridPlan& p, const Words4& r, bool finite)
{
    if (!finite) return quantize_group_to_grid<MODE>(v, p, r);
    uint4 o;
    o.x = quantize_finite_to_grid<MODE>(v.x, p, r.w[0]);
    o.y = quantize_finite_to_grid<MODE>(v.y, p, r.w[1]);
    o.z = quantize_finite_to_grid<MODE>(v.z, p, r.w[2]);
    o.w = quantize_finite_to_grid<MODE>(v.w, p, r.w[3]);
    return o;
}

// plan_is_finite agreed on by the wavefront (plans may differ from lane to lane).
template <int MODE>
__device__ __forceinline__ bool wave_plans_are_finite(const GridPlan& p)
{
    return __all(plan_is_finite<MODE>(p) ? 1 : 0) != 0;
}

// Geometry of the [outer, nblocks, inner] view.  A block's elements are numbered t = o * inner + i;
// element t of block b sits at flat index (o * nblocks + b) * inner + i.
struct BlockGeom {
    uint64_t n, outer, nblocks, inner;
};

}  // namespace qsim
