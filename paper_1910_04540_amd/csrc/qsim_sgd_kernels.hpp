// The fused quantized SGD-with-momentum step.
#pragma once

#include "qsim_kernel_common.hpp"

namespace qsim {

// ---------------------------------------------------------------------------------------------
// Fused quantized SGD step.  A workgroup walks tiles of 1024 elements (one group per thread), so a
// chunk of L <= 1024 elements never leaves the workgroup: its maximum is a reduction over L/4
// neighbouring lanes (inside a wave up to L = 256, through LDS above).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t chunk_max(uint32_t v, int lanes, uint32_t* lds)
{
    if (lanes <= 64) return group_max(v, lanes);
    // lanes is 128 or 256: whole waves
    const uint32_t w = wave_max(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[wave] = w;
    __syncthreads();
    if (lanes == 128) {
        const uint32_t a = lds[wave & ~1], b = lds[wave | 1];
        return a > b ? a : b;
    }
    uint32_t m = lds[0];
#pragma unroll
    for (int k = 1; k < kThreads / 64; ++k) m = m > lds[k] ? m : lds[k];
    return m;
}

// Quantize one group with a run-time format.  Called by every thread of the workgroup (a block
// kind synchronises inside); groups past the end of the array carry zeros.
__device__ __forceinline__ uint4 apply_format(const FormatPlan& f, const uint4& v, uint64_t j, const RngKey& key,
                                              uint32_t role, uint32_t* lds)
{
    if (f.kind == 0) return v;
    Words4 r = {{0u, 0u, 0u, 0u}};
    if (f.mode == QSIM_STOCHASTIC) r = random_words(j, key, role);
    if (f.kind == 3) {
        const GridPlan p = block_plan(chunk_max(max4_mag(v), f.lanes, lds), f.wl, f.symmetric);
        return quantize_group_rt(f, p, v, r);
    }
    return quantize_group_rt(f, f.grid, v, r);
}

__device__ __forceinline__ uint32_t fma_bits(float a, uint32_t b, uint32_t c)
{
    return __float_as_uint(__builtin_fmaf(a, __uint_as_float(b), __uint_as_float(c)));
}

// Scalars of the step (Sec. 3.1 "Front-end interface": the optimizer update the quantizers wrap).
struct SgdHyper {
    float lr, momentum;
    float weight_decay;   // used when has_decay
    float keep;           // 1 - dampening in fp32, used when has_dampening
    int has_decay, has_dampening, nesterov;
};

// One tile of 1024 elements of one tensor.  Called by every thread of the workgroup (a block kind
// synchronises inside); groups past the end of the array load zeros and store nothing.
// `w_q` may be NULL (no quantized copy) or equal to `w_master` (the weights themselves are kept in
// the weight format: only the quantized value is stored).
// Per element, every line one fp32 operation:
//   gq = Qg(g);  d = fma(weight_decay, w, gq);  v = Qm(fma(momentum, v, keep * d));
//   w = fma(-lr, nesterov ? fma(momentum, v, d) : v, w);  w_q = Qw(w)
// where the weight-decay, dampening and Nesterov terms are skipped when their option is off.
template <bool VEC>
__device__ __forceinline__ void sgd_tile(uint32_t* w_master, uint32_t* w_q, const uint32_t* grad, uint32_t* mom, uint64_t n,
                                         uint64_t tile, const SgdHyper& h, const FormatPlan& fg, const FormatPlan& fm,
                                         const FormatPlan& fw, const RngKey& key, uint32_t* lds)
{
    const uint64_t j = tile * kThreads + threadIdx.x;
    const uint4 g = load_group<VEC>(grad, j, n);
    const uint4 v = load_group<VEC>(mom, j, n);
    const uint4 w = load_group<VEC>(w_master, j, n);

    uint4 d = apply_format(fg, g, j, key, 0u, lds);
    if (h.has_decay) {
        d.x = fma_bits(h.weight_decay, w.x, d.x);
        d.y = fma_bits(h.weight_decay, w.y, d.y);
        d.z = fma_bits(h.weight_decay, w.z, d.z);
        d.w = fma_bits(h.weight_decay, w.w, d.w);
    }
    uint4 t = d;
    if (h.has_dampening) {
        t.x = __float_as_uint(h.keep * __uint_as_float(d.x));
        t.y = __float_as_uint(h.keep * __uint_as_float(d.y));
        t.z = __float_as_uint(h.keep * __uint_as_float(d.z));
        t.w = __float_as_uint(h.keep * __uint_as_float(d.w));
    }
    t.x = fma_bits(h.momentum, v.x, t.x);
    t.y = fma_bits(h.momentum, v.y, t.y);
    t.z = fma_bits(h.momentum, v.z, t.z);
    t.w = fma_bits(h.momentum, v.w, t.w);
    const uint4 vq = apply_format(fm, t, j, key, 1u, lds);
    uint4 step = vq;
    if (h.nesterov) {
        step.x = fma_bits(h.momentum, vq.x, d.x);
        step.y = fma_bits(h.momentum, vq.y, d.y);
        step.z = fma_bits(h.momentum, vq.z, d.z);
        step.w = fma_bits(h.momentum, vq.w, d.w);
    }
    uint4 wn;
    wn.x = fma_bits(-h.lr, step.x, w.x);
    wn.y = fma_bits(-h.lr, step.y, w.y);
    wn.z = fma_bits(-h.lr, step.z, w.z);
    wn.w = fma_bits(-h.lr, step.w, w.w);
    // elements past the end are zero up to here (zero loads, and every operation above maps zeros
    // to zero), so they cannot disturb a chunk maximum
    store_group<VEC>(mom, j, n, vq);
    if (w_q != w_master) store_group<VEC>(w_master, j, n, wn);
    if (w_q) store_group<VEC>(w_q, j, n, apply_format(fw, wn, j, key, 2u, lds));
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void sgd_step_kernel(uint32_t* w_master, uint32_t* w_q, const uint32_t* grad,
                                                            uint32_t* mom, uint64_t n, uint64_t tiles, SgdHyper h,
                                                            FormatPlan fg, FormatPlan fm, FormatPlan fw, RngKey key)
{
    __shared__ uint32_t lds[kThreads / 64];
    // every thread of a workgroup runs the same number of tiles, so the barriers inside
    // apply_format are reached by all of them
    for (uint64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x)
        sgd_tile<VEC>(w_master, w_q, grad, mom, n, tile, h, fg, fm, fw, key, lds);
}

// The same step over a list of tensors in one launch (a model's parameter tensors are many and
// mostly small, so one launch per tensor would be bound by launch latency).  The table travels in
// the kernel arguments; workgroup `blockIdx.x` finds its tensor from the running tile counts.
// Tensor t draws its random words from stream `key.stream_id + t`.
constexpr int kMultiTensors = 64;

struct MultiTensorTable {
    uint32_t* w_master[kMultiTensors];
    uint32_t* w_q[kMultiTensors];
    const uint32_t* grad[kMultiTensors];
    uint32_t* mom[kMultiTensors];
    uint64_t n[kMultiTensors];
    uint32_t first_tile[kMultiTensors + 1];     // running sum of tiles
    int count;
};

template <bool VEC>
__global__ __launch_bounds__(kThreads) void sgd_multi_kernel(MultiTensorTable tab, SgdHyper h, FormatPlan fg, FormatPlan fm,
                                                             FormatPlan fw, RngKey key)
{
    __shared__ uint32_t lds[kThreads / 64];
    const uint32_t tile = (uint32_t)linear_block();
    if (tile >= tab.first_tile[tab.count]) return;     // the whole workgroup leaves together
    int t = 0;
    while (t + 1 < tab.count && tile >= tab.first_tile[t + 1]) ++t;     // wave-uniform scan of at most 64 entries
    RngKey k = key;
    k.stream_id = key.stream_id + (uint32_t)t;
    sgd_tile<VEC>(tab.w_master[t], tab.w_q[t], tab.grad[t], tab.mom[t], tab.n[t], tile - tab.first_tile[t], h, fg, fm, fw, k,
                  lds);
}

// The same step over a list of any length, in one launch: the table lives in device memory
// (written once by the host for a fixed list of tensors, as an optimizer's is) instead of the
// kernel arguments.  `owner[tile]` names the entry a tile of 1024 elements belongs to, so a
// workgroup finds its tensor with two dependent uniform loads, whatever the length of the list.
struct SgdTableEntry {
    uint32_t* w_master;
    uint32_t* w_q;
    const uint32_t* grad;
    uint32_t* mom;
    uint64_t n;
    uint32_t first_tile;    // number of tiles of the entries before this one
    uint32_t position;      // index of the tensor in the caller's list: added to the stream id
};
static_assert(sizeof(SgdTableEntry) == 48, "the host lays the table out by this size");

template <bool VEC>
__global__ __launch_bounds__(kThreads) void sgd_table_kernel(const SgdTableEntry* __restrict__ entries,
                                                             const uint32_t* __restrict__ owner, uint32_t tiles, SgdHyper h,
                                                             FormatPlan fg, FormatPlan fm, FormatPlan fw, RngKey key)
{
    __shared__ uint32_t lds[kThreads / 64];
    const uint64_t tile = linear_block();
    if (tile >= tiles) return;     // the whole workgroup leaves together
    const SgdTableEntry e = entries[owner[tile]];
    RngKey k = key;
    k.stream_id = key.stream_id + e.position;
    sgd_tile<VEC>(e.w_master, e.w_q, e.grad, e.mom, e.n, tile - e.first_tile, h, fg, fm, fw, k, lds);
}

}  // namespace qsim
