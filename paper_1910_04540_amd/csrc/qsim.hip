// libqsim: entry points and kernels.  Hand-written HIP for gfx950 (MI355X); see include/qsim.h
// for the contract of every entry point.
//
// All kernels are streaming, HBM-bound bit manipulation: a thread's unit of work is one group of
// four consecutive elements whose first index is a multiple of four, i.e. one dwordx4 load, one
// Philox4x32-10 block (its four words belong to exactly these four elements) and one dwordx4
// store.  Arrays that are not 16-byte aligned take the same path with dword accesses.
#include <hip/hip_runtime.h>

#include "qsim.h"
#include "qsim_device.hpp"
#include "qsim_host.hpp"

namespace qsim {

constexpr int kThreads = 256;

// ---------------------------------------------------------------------------------------------
// Group access: elements [4*j, 4*j+4) of an array of n elements.
// ---------------------------------------------------------------------------------------------
template <bool VEC>
__device__ __forceinline__ uint4 load_group(const uint32_t* p, uint64_t j, uint64_t n)
{
    const uint64_t i = j * 4;
    if (VEC && i + 4 <= n) return *reinterpret_cast<const uint4*>(p + i);
    uint4 v = {0u, 0u, 0u, 0u};
    if (i + 0 < n) v.x = p[i + 0];
    if (i + 1 < n) v.y = p[i + 1];
    if (i + 2 < n) v.z = p[i + 2];
    if (i + 3 < n) v.w = p[i + 3];
    return v;
}

template <bool VEC>
__device__ __forceinline__ void store_group(uint32_t* p, uint64_t j, uint64_t n, const uint4& v)
{
    const uint64_t i = j * 4;
    if (VEC && i + 4 <= n) {
        *reinterpret_cast<uint4*>(p + i) = v;
        return;
    }
    if (i + 0 < n) p[i + 0] = v.x;
    if (i + 1 < n) p[i + 1] = v.y;
    if (i + 2 < n) p[i + 2] = v.z;
    if (i + 3 < n) p[i + 3] = v.w;
}

struct RngKey {
    uint32_t seed_lo, seed_hi, stream_id;
};

// ---------------------------------------------------------------------------------------------
// Elementwise quantizers (fixed point, floating point).
// ---------------------------------------------------------------------------------------------
struct FixedOp {
    GridPlan plan;
    template <int MODE>
    __device__ __forceinline__ uint32_t apply(uint32_t bits, uint32_t r) const
    {
        return quantize_to_grid<MODE>(bits, plan, r);
    }
};

struct FloatOp {
    FloatPlan plan;
    template <int MODE>
    __device__ __forceinline__ uint32_t apply(uint32_t bits, uint32_t r) const
    {
        return quantize_float<MODE>(bits, plan, r);
    }
};

template <class Op, int MODE, bool VEC, int UNROLL>
__global__ __launch_bounds__(kThreads) void elementwise_kernel(const uint32_t* in, uint32_t* out, uint64_t n,
                                                               uint64_t groups, Op op, RngKey key)
{
    const uint64_t base = (uint64_t)blockIdx.x * (kThreads * UNROLL) + threadIdx.x;
    uint4 v[UNROLL];
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint64_t j = base + (uint64_t)k * kThreads;
        if (j < groups) v[k] = load_group<VEC>(in, j, n);
    }
#pragma unroll
    for (int k = 0; k < UNROLL; ++k) {
        const uint64_t j = base + (uint64_t)k * kThreads;
        if (j < groups) {
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (MODE == QSIM_STOCHASTIC) r = random_words(j, key.seed_lo, key.seed_hi, key.stream_id, 0u);
            uint4 o;
            o.x = op.template apply<MODE>(v[k].x, r.w[0]);
            o.y = op.template apply<MODE>(v[k].y, r.w[1]);
            o.z = op.template apply<MODE>(v[k].z, r.w[2]);
            o.w = op.template apply<MODE>(v[k].w, r.w[3]);
            store_group<VEC>(out, j, n, o);
        }
    }
}

template <class Op, int MODE, bool VEC>
static int launch_elementwise_mode(const float* in, float* out, uint64_t n, const Op& op, const RngKey& key,
                                   hipStream_t stream)
{
    constexpr int UNROLL = 4;
    const uint64_t groups = (n + 3) / 4;
    const uint64_t blocks = (groups + kThreads * UNROLL - 1) / (kThreads * UNROLL);
    hipLaunchKernelGGL((elementwise_kernel<Op, MODE, VEC, UNROLL>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                       reinterpret_cast<const uint32_t*>(in), reinterpret_cast<uint32_t*>(out), n, groups, op, key);
    return hipGetLastError() == hipSuccess ? QSIM_OK : QSIM_ERR_LAUNCH;
}

template <class Op, bool VEC>
static int launch_elementwise_vec(const float* in, float* out, uint64_t n, int rounding, const Op& op,
                                  const RngKey& key, hipStream_t stream)
{
    switch (rounding) {
    case QSIM_RN_EVEN: return launch_elementwise_mode<Op, QSIM_RN_EVEN, VEC>(in, out, n, op, key, stream);
    case QSIM_RN_AWAY: return launch_elementwise_mode<Op, QSIM_RN_AWAY, VEC>(in, out, n, op, key, stream);
    case QSIM_RN_ZERO: return launch_elementwise_mode<Op, QSIM_RN_ZERO, VEC>(in, out, n, op, key, stream);
    default:           return launch_elementwise_mode<Op, QSIM_STOCHASTIC, VEC>(in, out, n, op, key, stream);
    }
}

template <class Op>
static int launch_elementwise(const float* in, float* out, uint64_t n, int rounding, const Op& op, const RngKey& key,
                              hipStream_t stream)
{
    if (aligned16(in) && aligned16(out)) return launch_elementwise_vec<Op, true>(in, out, n, rounding, op, key, stream);
    return launch_elementwise_vec<Op, false>(in, out, n, rounding, op, key, stream);
}

// ---------------------------------------------------------------------------------------------
// Block floating point.
//
// Workgroup-wide maximum: wave reduction, then one LDS slot per wave.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t workgroup_max(uint32_t v, uint32_t* lds /* kThreads/64 + 1 slots */)
{
    const uint32_t w = wave_max(v);
    const int wave = threadIdx.x >> 6;
    __syncthreads();                        // protects the slots against the previous use
    if ((threadIdx.x & 63) == 0) lds[wave] = w;
    __syncthreads();
    uint32_t m = lds[0];
#pragma unroll
    for (int k = 1; k < kThreads / 64; ++k) m = m > lds[k] ? m : lds[k];
    return m;
}

// Geometry of the [outer, nblocks, inner] view.  A block's elements are numbered t = o * inner + i;
// element t of block b sits at flat index (o * nblocks + b) * inner + i.
struct BlockGeom {
    uint64_t n, outer, nblocks, inner;
};

// One contiguous block per workgroup (outer == 1): the block is read twice by the same workgroup,
// the second time out of cache, so HBM sees it once.  VEC needs inner % 4 == 0 and aligned arrays.
template <int MODE, bool VEC>
__global__ __launch_bounds__(kThreads) void block_rows_kernel(const uint32_t* in, uint32_t* out, BlockGeom g, int wl,
                                                              int symmetric, RngKey key)
{
    __shared__ uint32_t lds[kThreads / 64];
    const uint64_t b = blockIdx.x;
    const uint64_t start = b * g.inner;
    const uint64_t len = (g.n - start < g.inner) ? g.n - start : g.inner;
    uint32_t m = 0;
    if (VEC) {
        // start is a multiple of four, so groups are those of the whole array
        const uint64_t j0 = start / 4, groups = (len + 3) / 4;
        for (uint64_t t = threadIdx.x; t < groups; t += kThreads) {
            const uint32_t gm = max4_mag(load_group<true>(in, j0 + t, start + len));
            m = m > gm ? m : gm;
        }
        const GridPlan p = block_plan(workgroup_max(m, lds), wl, symmetric);
        for (uint64_t t = threadIdx.x; t < groups; t += kThreads) {
            const uint64_t j = j0 + t;
            const uint4 v = load_group<true>(in, j, start + len);
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (MODE == QSIM_STOCHASTIC) r = random_words(j, key.seed_lo, key.seed_hi, key.stream_id, 0u);
            uint4 o;
            o.x = quantize_to_grid<MODE>(v.x, p, r.w[0]);
            o.y = quantize_to_grid<MODE>(v.y, p, r.w[1]);
            o.z = quantize_to_grid<MODE>(v.z, p, r.w[2]);
            o.w = quantize_to_grid<MODE>(v.w, p, r.w[3]);
            store_group<true>(out, j, start + len, o);
        }
    } else {
        for (uint64_t t = threadIdx.x; t < len; t += kThreads) {
            const uint32_t a = in[start + t] & 0x7fffffffu;
            m = m > a ? m : a;
        }
        const GridPlan p = block_plan(workgroup_max(m, lds), wl, symmetric);
        for (uint64_t t = threadIdx.x; t < len; t += kThreads) {
            const uint64_t i = start + t;
            uint32_t r = 0;
            if (MODE == QSIM_STOCHASTIC) r = random_words(i >> 2, key.seed_lo, key.seed_hi, key.stream_id, 0u).w[i & 3];
            out[i] = quantize_to_grid<MODE>(in[i], p, r);
        }
    }
}

// Blocks spread over several workgroups, any layout.  Pass 1: workgroup (b, s) reduces slice s of
// block b and writes one partial maximum to partial[b * slices + s] (no atomics, so the scratch
// needs no initialisation).  Pass 2: every workgroup folds the partials of its block, then
// quantizes its slice.  A slice is a range of t = o * inner + i.
// VEC: inner % 4 == 0 and aligned arrays, so four consecutive t are four consecutive addresses.
struct SliceGeom {
    BlockGeom g;
    uint64_t block_len;    // outer * inner (for outer == 1 the last block may be shorter)
    uint64_t slice_len;    // elements of t per workgroup, a multiple of 4
    uint32_t slices;       // workgroups per block
};

__device__ __forceinline__ uint64_t flat_index(const BlockGeom& g, uint64_t b, uint64_t t)
{
    if (g.outer == 1) return b * g.inner + t;
    const uint64_t o = t / g.inner, i = t - o * g.inner;
    return (o * g.nblocks + b) * g.inner + i;
}

__device__ __forceinline__ uint64_t block_length(const SliceGeom& sg, uint64_t b)
{
    if (sg.g.outer != 1) return sg.block_len;
    const uint64_t start = b * sg.g.inner;
    return (sg.g.n - start < sg.g.inner) ? sg.g.n - start : sg.g.inner;
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void block_partial_max_kernel(const uint32_t* in, uint32_t* partial, SliceGeom sg)
{
    __shared__ uint32_t lds[kThreads / 64];
    const uint64_t b = blockIdx.x;
    const uint64_t len = block_length(sg, b);
    const uint64_t t0 = (uint64_t)blockIdx.y * sg.slice_len;
    const uint64_t t1 = (t0 + sg.slice_len < len) ? t0 + sg.slice_len : len;
    uint32_t m = 0;
    if (VEC) {
        for (uint64_t t = t0 + 4ull * threadIdx.x; t < t1; t += 4ull * kThreads) {
            const uint64_t i = flat_index(sg.g, b, t);
            const uint32_t gm = max4_mag(load_group<true>(in, i / 4, sg.g.n));
            m = m > gm ? m : gm;
        }
    } else {
        for (uint64_t t = t0 + threadIdx.x; t < t1; t += kThreads) {
            const uint32_t a = in[flat_index(sg.g, b, t)] & 0x7fffffffu;
            m = m > a ? m : a;
        }
    }
    m = workgroup_max(m, lds);
    if (threadIdx.x == 0) partial[b * sg.slices + blockIdx.y] = m;
}

template <int MODE, bool VEC>
__global__ __launch_bounds__(kThreads) void block_apply_kernel(const uint32_t* in, uint32_t* out, const uint32_t* partial,
                                                               SliceGeom sg, int wl, int symmetric, RngKey key)
{
    __shared__ uint32_t lds[kThreads / 64];
    const uint64_t b = blockIdx.x;
    uint32_t m = 0;
    for (uint32_t s = threadIdx.x; s < sg.slices; s += kThreads) {
        const uint32_t a = partial[b * sg.slices + s];
        m = m > a ? m : a;
    }
    const GridPlan p = block_plan(workgroup_max(m, lds), wl, symmetric);
    const uint64_t len = block_length(sg, b);
    const uint64_t t0 = (uint64_t)blockIdx.y * sg.slice_len;
    const uint64_t t1 = (t0 + sg.slice_len < len) ? t0 + sg.slice_len : len;
    if (VEC) {
        for (uint64_t t = t0 + 4ull * threadIdx.x; t < t1; t += 4ull * kThreads) {
            const uint64_t j = flat_index(sg.g, b, t) / 4;
            const uint4 v = load_group<true>(in, j, sg.g.n);
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (MODE == QSIM_STOCHASTIC) r = random_words(j, key.seed_lo, key.seed_hi, key.stream_id, 0u);
            uint4 o;
            o.x = quantize_to_grid<MODE>(v.x, p, r.w[0]);
            o.y = quantize_to_grid<MODE>(v.y, p, r.w[1]);
            o.z = quantize_to_grid<MODE>(v.z, p, r.w[2]);
            o.w = quantize_to_grid<MODE>(v.w, p, r.w[3]);
            store_group<true>(out, j, sg.g.n, o);
        }
    } else {
        for (uint64_t t = t0 + threadIdx.x; t < t1; t += kThreads) {
            const uint64_t i = flat_index(sg.g, b, t);
            uint32_t r = 0;
            if (MODE == QSIM_STOCHASTIC) r = random_words(i >> 2, key.seed_lo, key.seed_hi, key.stream_id, 0u).w[i & 3];
            out[i] = quantize_to_grid<MODE>(in[i], p, r);
        }
    }
}

// How a block-quantize call is carried out; decided on the host from the shape alone, so that
// qsim_block_workspace_bytes and qsim_block_quantize always agree.
struct BlockSchedule {
    bool rows;             // one workgroup per contiguous block, single launch
    SliceGeom sg;          // otherwise: two launches over slices
    size_t workspace;      // bytes of scratch needed
};

constexpr uint64_t kRowsMinInner = 1;            // below this a workgroup per block wastes lanes
constexpr uint64_t kRowsMaxInner = 1ull << 16;   // a block up to 256 KiB is re-read out of cache
constexpr uint32_t kMaxSlices = 1024;
constexpr uint64_t kMinSliceLen = 8192;

static BlockSchedule block_schedule(uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner)
{
    BlockSchedule s;
    memset(&s, 0, sizeof(s));
    s.sg.g = BlockGeom{n, outer, nblocks, inner};
    s.sg.block_len = outer * inner;
    // enough blocks to fill the chip, each small enough to stay in cache between the two reads
    s.rows = (outer == 1 && inner >= kRowsMinInner && inner <= kRowsMaxInner && nblocks >= 512) ||
             (outer == 1 && inner <= 4096);
    if (s.rows) return s;
    uint64_t slices = (s.sg.block_len + kMinSliceLen - 1) / kMinSliceLen;
    if (slices > kMaxSlices) slices = kMaxSlices;
    uint64_t slice_len = (s.sg.block_len + slices - 1) / slices;
    slice_len = (slice_len + 1023) / 1024 * 1024;
    slices = (s.sg.block_len + slice_len - 1) / slice_len;
    s.sg.slice_len = slice_len;
    s.sg.slices = (uint32_t)slices;
    s.workspace = (size_t)(nblocks * slices * sizeof(uint32_t));
    return s;
}

template <int MODE>
static int launch_block_mode(const float* in, float* out, const BlockSchedule& s, int wl, int symmetric,
                             const RngKey& key, void* workspace, hipStream_t stream)
{
    const uint32_t* pin = reinterpret_cast<const uint32_t*>(in);
    uint32_t* pout = reinterpret_cast<uint32_t*>(out);
    const BlockGeom& g = s.sg.g;
    const bool vec = aligned16(in) && aligned16(out) && (g.inner % 4 == 0);
    if (s.rows) {
        if (vec)
            hipLaunchKernelGGL((block_rows_kernel<MODE, true>), dim3((unsigned)g.nblocks), dim3(kThreads), 0, stream, pin,
                               pout, g, wl, symmetric, key);
        else
            hipLaunchKernelGGL((block_rows_kernel<MODE, false>), dim3((unsigned)g.nblocks), dim3(kThreads), 0, stream, pin,
                               pout, g, wl, symmetric, key);
        return hipGetLastError() == hipSuccess ? QSIM_OK : QSIM_ERR_LAUNCH;
    }
    uint32_t* partial = reinterpret_cast<uint32_t*>(workspace);
    const dim3 grid((unsigned)g.nblocks, s.sg.slices);
    if (vec) {
        hipLaunchKernelGGL((block_partial_max_kernel<true>), grid, dim3(kThreads), 0, stream, pin, partial, s.sg);
        hipLaunchKernelGGL((block_apply_kernel<MODE, true>), grid, dim3(kThreads), 0, stream, pin, pout, partial, s.sg, wl,
                           symmetric, key);
    } else {
        hipLaunchKernelGGL((block_partial_max_kernel<false>), grid, dim3(kThreads), 0, stream, pin, partial, s.sg);
        hipLaunchKernelGGL((block_apply_kernel<MODE, false>), grid, dim3(kThreads), 0, stream, pin, pout, partial, s.sg, wl,
                           symmetric, key);
    }
    return hipGetLastError() == hipSuccess ? QSIM_OK : QSIM_ERR_LAUNCH;
}

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

__device__ __forceinline__ uint32_t apply_scalar_format(const FormatPlan& f, uint32_t bits, uint32_t r)
{
    if (f.kind == 1) {
        switch (f.mode) {
        case QSIM_RN_EVEN: return quantize_float<QSIM_RN_EVEN>(bits, f.flt, r);
        case QSIM_RN_AWAY: return quantize_float<QSIM_RN_AWAY>(bits, f.flt, r);
        case QSIM_RN_ZERO: return quantize_float<QSIM_RN_ZERO>(bits, f.flt, r);
        default:           return quantize_float<QSIM_STOCHASTIC>(bits, f.flt, r);
        }
    }
    return bits;
}

__device__ __forceinline__ uint32_t apply_grid_rt(int mode, uint32_t bits, const GridPlan& p, uint32_t r)
{
    switch (mode) {
    case QSIM_RN_EVEN: return quantize_to_grid<QSIM_RN_EVEN>(bits, p, r);
    case QSIM_RN_AWAY: return quantize_to_grid<QSIM_RN_AWAY>(bits, p, r);
    case QSIM_RN_ZERO: return quantize_to_grid<QSIM_RN_ZERO>(bits, p, r);
    default:           return quantize_to_grid<QSIM_STOCHASTIC>(bits, p, r);
    }
}

// Quantize one group with a run-time format.  Called by every thread of the workgroup (a block
// kind synchronises inside); `live` is false for threads past the end, whose values are zero.
__device__ __forceinline__ uint4 apply_format(const FormatPlan& f, uint4 v, uint64_t j, const RngKey& key, uint32_t role,
                                              uint32_t* lds)
{
    if (f.kind == 0) return v;
    Words4 r = {{0u, 0u, 0u, 0u}};
    if (f.mode == QSIM_STOCHASTIC) r = random_words(j, key.seed_lo, key.seed_hi, key.stream_id, role);
    uint4 o;
    if (f.kind == 1) {
        o.x = apply_scalar_format(f, v.x, r.w[0]);
        o.y = apply_scalar_format(f, v.y, r.w[1]);
        o.z = apply_scalar_format(f, v.z, r.w[2]);
        o.w = apply_scalar_format(f, v.w, r.w[3]);
        return o;
    }
    GridPlan p = f.grid;
    if (f.kind == 3) p = block_plan(chunk_max(max4_mag(v), f.lanes, lds), f.wl, f.symmetric);
    o.x = apply_grid_rt(f.mode, v.x, p, r.w[0]);
    o.y = apply_grid_rt(f.mode, v.y, p, r.w[1]);
    o.z = apply_grid_rt(f.mode, v.z, p, r.w[2]);
    o.w = apply_grid_rt(f.mode, v.w, p, r.w[3]);
    return o;
}

__device__ __forceinline__ uint32_t fma_bits(float a, uint32_t b, uint32_t c)
{
    return __float_as_uint(__builtin_fmaf(a, __uint_as_float(b), __uint_as_float(c)));
}

template <bool VEC>
__global__ __launch_bounds__(kThreads) void sgd_step_kernel(uint32_t* w_master, uint32_t* w_q, const uint32_t* grad,
                                                            uint32_t* mom, uint64_t n, uint64_t tiles, float lr,
                                                            float momentum, FormatPlan fg, FormatPlan fm, FormatPlan fw,
                                                            RngKey key)
{
    __shared__ uint32_t lds[kThreads / 64];
    // every thread of a workgroup runs the same number of tiles, so the barriers inside
    // apply_format are reached by all of them; groups past the end load zeros and store nothing
    for (uint64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const uint64_t j = tile * kThreads + threadIdx.x;
        const uint4 g = load_group<VEC>(grad, j, n);
        const uint4 v = load_group<VEC>(mom, j, n);
        const uint4 w = load_group<VEC>(w_master, j, n);

        const uint4 gq = apply_format(fg, g, j, key, 0u, lds);
        uint4 t;
        t.x = fma_bits(momentum, v.x, gq.x);
        t.y = fma_bits(momentum, v.y, gq.y);
        t.z = fma_bits(momentum, v.z, gq.z);
        t.w = fma_bits(momentum, v.w, gq.w);
        // lanes past the end must not disturb a chunk maximum: their fma result is forced to zero
        const uint64_t i = j * 4;
        if (i + 0 >= n) t.x = 0u;
        if (i + 1 >= n) t.y = 0u;
        if (i + 2 >= n) t.z = 0u;
        if (i + 3 >= n) t.w = 0u;
        const uint4 vq = apply_format(fm, t, j, key, 1u, lds);
        uint4 wn;
        wn.x = fma_bits(-lr, vq.x, w.x);
        wn.y = fma_bits(-lr, vq.y, w.y);
        wn.z = fma_bits(-lr, vq.z, w.z);
        wn.w = fma_bits(-lr, vq.w, w.w);
        if (i + 0 >= n) wn.x = 0u;
        if (i + 1 >= n) wn.y = 0u;
        if (i + 2 >= n) wn.z = 0u;
        if (i + 3 >= n) wn.w = 0u;
        store_group<VEC>(mom, j, n, vq);
        store_group<VEC>(w_master, j, n, wn);
        if (w_q) {
            const uint4 wq = apply_format(fw, wn, j, key, 2u, lds);
            store_group<VEC>(w_q, j, n, wq);
        }
    }
}

static hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

}  // namespace qsim

using namespace qsim;

extern "C" {

int qsim_float_quantize(const float* in, float* out, uint64_t n, int exp_bits, int man_bits, int rounding,
                        uint32_t flags, uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    if (!valid_rounding(rounding)) return QSIM_ERR_ROUNDING;
    if (!valid_float(exp_bits, man_bits) || !valid_flags(flags)) return QSIM_ERR_FORMAT;
    if (n > kMaxElements) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!in || !out) return QSIM_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_ERR_OVERLAP;
    const FloatOp op{float_plan(exp_bits, man_bits, flags)};
    const RngKey key{(uint32_t)seed, (uint32_t)(seed >> 32), stream_id};
    return launch_elementwise(in, out, n, rounding, op, key, as_stream(hip_stream));
}

int qsim_fixed_quantize(const float* in, float* out, uint64_t n, int wl, int fl, int rounding, uint32_t flags,
                        uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    if (!valid_rounding(rounding)) return QSIM_ERR_ROUNDING;
    if (!valid_fixed(wl, fl) || !valid_flags(flags)) return QSIM_ERR_FORMAT;
    if (n > kMaxElements) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!in || !out) return QSIM_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_ERR_OVERLAP;
    const FixedOp op{fixed_plan(wl, fl, flags)};
    const RngKey key{(uint32_t)seed, (uint32_t)(seed >> 32), stream_id};
    return launch_elementwise(in, out, n, rounding, op, key, as_stream(hip_stream));
}

size_t qsim_block_workspace_bytes(uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner)
{
    if (n == 0 || n > kMaxElements || !valid_block_shape(n, outer, nblocks, inner)) return 0;
    return block_schedule(n, outer, nblocks, inner).workspace;
}

int qsim_block_quantize(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner,
                        int wl, int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id, void* workspace,
                        size_t workspace_bytes, void* hip_stream)
{
    if (!valid_rounding(rounding)) return QSIM_ERR_ROUNDING;
    if (!valid_block_wl(wl) || !valid_flags(flags)) return QSIM_ERR_FORMAT;
    if (n > kMaxElements) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!valid_block_shape(n, outer, nblocks, inner)) return QSIM_ERR_SHAPE;
    if (!in || !out) return QSIM_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_ERR_OVERLAP;
    const BlockSchedule s = block_schedule(n, outer, nblocks, inner);
    if (nblocks > 0x7fffffffull) return QSIM_ERR_UNSUPPORTED;
    if (s.workspace) {
        if (!workspace || !aligned16(workspace) || workspace_bytes < s.workspace) return QSIM_ERR_WORKSPACE;
        if (any_overlap(workspace, in, n) || any_overlap(workspace, out, n)) return QSIM_ERR_OVERLAP;
    }
    const RngKey key{(uint32_t)seed, (uint32_t)(seed >> 32), stream_id};
    const int symmetric = (flags & QSIM_SYMMETRIC) ? 1 : 0;
    hipStream_t stream = as_stream(hip_stream);
    switch (rounding) {
    case QSIM_RN_EVEN: return launch_block_mode<QSIM_RN_EVEN>(in, out, s, wl, symmetric, key, workspace, stream);
    case QSIM_RN_AWAY: return launch_block_mode<QSIM_RN_AWAY>(in, out, s, wl, symmetric, key, workspace, stream);
    case QSIM_RN_ZERO: return launch_block_mode<QSIM_RN_ZERO>(in, out, s, wl, symmetric, key, workspace, stream);
    default:           return launch_block_mode<QSIM_STOCHASTIC>(in, out, s, wl, symmetric, key, workspace, stream);
    }
}

int qsim_quant_sgd_step(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n, float lr,
                        float momentum, const qsim_format* fmt_grad, const qsim_format* fmt_mom,
                        const qsim_format* fmt_weight, uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    FormatPlan fg, fm, fw;
    int status;
    if ((status = make_format_plan(fmt_grad, &fg)) != QSIM_OK) return status;
    if ((status = make_format_plan(fmt_mom, &fm)) != QSIM_OK) return status;
    if ((status = make_format_plan(fmt_weight, &fw)) != QSIM_OK) return status;
    if (n > kMaxElements) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!w_master || !grad || !mom) return QSIM_ERR_NULL;
    if (any_overlap(w_master, grad, n) || any_overlap(w_master, mom, n) || any_overlap(grad, mom, n))
        return QSIM_ERR_OVERLAP;
    if (w_q && (any_overlap(w_q, w_master, n) || any_overlap(w_q, grad, n) || any_overlap(w_q, mom, n)))
        return QSIM_ERR_OVERLAP;
    const RngKey key{(uint32_t)seed, (uint32_t)(seed >> 32), stream_id};
    const uint64_t groups = (n + 3) / 4;
    const uint64_t tiles = (groups + kThreads - 1) / kThreads;
    const unsigned blocks = (unsigned)(tiles < 0x7fffffffull ? tiles : 0x7fffffffull);
    const bool vec = aligned16(w_master) && aligned16(grad) && aligned16(mom) && (!w_q || aligned16(w_q));
    uint32_t* pw = reinterpret_cast<uint32_t*>(w_master);
    uint32_t* pq = reinterpret_cast<uint32_t*>(w_q);
    const uint32_t* pg = reinterpret_cast<const uint32_t*>(grad);
    uint32_t* pm = reinterpret_cast<uint32_t*>(mom);
    if (vec)
        hipLaunchKernelGGL((sgd_step_kernel<true>), dim3(blocks), dim3(kThreads), 0, as_stream(hip_stream), pw, pq, pg, pm,
                           n, tiles, lr, momentum, fg, fm, fw, key);
    else
        hipLaunchKernelGGL((sgd_step_kernel<false>), dim3(blocks), dim3(kThreads), 0, as_stream(hip_stream), pw, pq, pg, pm,
                           n, tiles, lr, momentum, fg, fm, fw, key);
    return hipGetLastError() == hipSuccess ? QSIM_OK : QSIM_ERR_LAUNCH;
}

const char* qsim_status_string(int status)
{
    switch (status) {
    case QSIM_OK: return "ok";
    case QSIM_ERR_NULL: return "a required pointer is NULL";
    case QSIM_ERR_FORMAT: return "format parameters or flags out of range";
    case QSIM_ERR_ROUNDING: return "unknown rounding mode";
    case QSIM_ERR_SHAPE: return "element count does not match the block layout or is too large";
    case QSIM_ERR_OVERLAP: return "arrays overlap";
    case QSIM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case QSIM_ERR_UNSUPPORTED: return "unsupported configuration";
    case QSIM_ERR_LAUNCH: return "the HIP runtime refused the launch";
    default: return "unknown status";
    }
}

}  // extern "C"
