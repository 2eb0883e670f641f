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

// ---------------------------------------------------------------------------------------------
// Block floating point.
// ---------------------------------------------------------------------------------------------

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

// Geometry of the [outer, nblocks, inner] view.  A block's elements are numbered t = o * inner + i;
// element t of block b sits at flat index (o * nblocks + b) * inner + i.
struct BlockGeom {
    uint64_t n, outer, nblocks, inner;
};

// Contiguous blocks (outer == 1, inner % 4 == 0, aligned arrays) held in registers: a team of
// `team` lanes (a power of two, 1..64) or the whole workgroup of THREADS threads owns one block and
// every lane keeps GPT groups of it, so the block is read from memory exactly once.
// Requires ceil(inner / 4) <= team * GPT (THREADS * GPT for the whole workgroup).  With 16 groups
// per thread (128 registers per lane) 512 threads hold a block of 32,768 elements and 1024 threads
// one of 65,536: a quarter and a half of a compute unit's registers.
template <int MODE, int GPT, bool WHOLE_WORKGROUP, int THREADS = kThreads>
__global__ __launch_bounds__(THREADS) void block_cached_kernel(const uint32_t* in, uint32_t* out, BlockGeom g,
                                                               int team_log2, int wl, int symmetric, RngKey key)
{
    __shared__ uint32_t lds[THREADS / 64];
    const int team = 1 << team_log2;
    const uint32_t teams_per_wg = WHOLE_WORKGROUP ? 1u : (uint32_t)(THREADS >> team_log2);
    // Everything a lane needs is a 32-bit offset from the workgroup's first element, which is
    // wave-uniform: the 64-bit arithmetic stays in scalar registers.
    const uint64_t b0 = linear_block() * teams_per_wg;              // first block of the workgroup
    if (b0 >= g.nblocks) return;                                    // the whole workgroup leaves together
    const uint64_t e0 = b0 * g.inner;                               // its first element (a multiple of four)
    const uint32_t* win = in + e0;
    uint32_t* wout = out + e0;
    const uint64_t left = g.n - e0;
    const uint32_t avail = left < 0x40000000ull ? (uint32_t)left : 0x40000000u;     // elements up to the array's end
    const uint32_t inner = (uint32_t)g.inner;                       // at most 65,536 here
    const uint32_t lane = WHOLE_WORKGROUP ? threadIdx.x : (threadIdx.x & (uint32_t)(team - 1));
    const uint32_t first = WHOLE_WORKGROUP ? 0u : (threadIdx.x >> team_log2) * inner;   // the team's block, relative
    // a team past the last block keeps all its lanes running with nothing to load or store, so the
    // cross-lane operations below always see a full wavefront; the last block may be short
    const uint32_t len = first >= avail ? 0u : (avail - first < inner ? avail - first : inner);
    const uint32_t end = first + len;
    const uint32_t g0 = first / 4u;
    const uint32_t groups = (len + 3u) / 4u;
    const uint32_t stride = WHOLE_WORKGROUP ? (uint32_t)THREADS : (uint32_t)team;
    const uint64_t j0 = e0 / 4;                                     // uniform: the workgroup's first group

    uint4 v[GPT];
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = lane + (uint32_t)k * stride;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        if (t < groups) v[k] = load_group<true>(win, (uint64_t)(g0 + t), (uint64_t)end);
    }
    // stochastic rounding: the random words of the first groups are drawn while the loads are in
    // flight (they do not depend on the data), the rest after the reduction
    // (the large workgroups have 128 registers per lane, half of them data: fewer words drawn early, not pinned)
    constexpr int kEarly = THREADS > kThreads ? 4 : 8;
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? (GPT < kEarly ? GPT : kEarly) : 0;
    Words4 early[PRE > 0 ? PRE : 1];
#pragma unroll
    for (int k = 0; k < PRE; ++k) {
        early[k] = random_words(j0 + (g0 + lane + (uint32_t)k * stride), key, 0u);
        // keep the compiler from sinking this below the reduction, where it would no longer overlap the loads
        if (THREADS <= kThreads)
            asm volatile("" : "+v"(early[k].w[0]), "+v"(early[k].w[1]), "+v"(early[k].w[2]), "+v"(early[k].w[3]));
    }
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t gm = max4_mag(v[k]);
        m = m > gm ? m : gm;
    }
    m = WHOLE_WORKGROUP ? workgroup_max<THREADS>(m, lds) : group_max(m, team);
    const GridPlan p = block_plan(m, wl, symmetric);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = lane + (uint32_t)k * stride;
        if (t < groups) {
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) r = early[k];
            else if (MODE == QSIM_STOCHASTIC) r = random_words(j0 + (g0 + t), key, 0u);
            store_group<true>(wout, (uint64_t)(g0 + t), (uint64_t)end, quantize_group_to_grid<MODE>(v[k], p, r));
        }
    }
}

// Contiguous blocks (outer == 1) of ANY length up to 4 * kThreads * GPT - 6, aligned arrays or not:
// the form for block lengths that are not a multiple of four (a 3x3 kernel's 27 weights, a row of
// 1001).  A workgroup owns `rows_per_wg` whole consecutive blocks, i.e. one contiguous range of
// elements, and walks it in the tensor's own groups of four (which is what the random words are
// keyed by, and what a dwordx4 access needs); a group may straddle blocks, and the first and last
// group of the range may be shared with the neighbouring workgroups, which each store only their
// own elements of it.  Block maxima meet in LDS (one ds_max per run of same-block elements of a
// group); every element then takes the plan of its own block.  The data is read once.
// `magic` = floor(2^32 / inner) + 1 (any value when inner == 1): element offset / inner by one
// multiply-high, exact for offsets below 2^16.
constexpr int kRaggedMaxRows = 4096;

template <int MODE, int GPT, bool VEC>
__global__ __launch_bounds__(kThreads) void block_ragged_kernel(const uint32_t* in, uint32_t* out, BlockGeom g,
                                                                uint32_t rows_per_wg, uint32_t magic, int wl, int symmetric,
                                                                RngKey key)
{
    __shared__ uint32_t rowmax[kRaggedMaxRows];
    const uint64_t r0 = linear_block() * rows_per_wg;
    if (r0 >= g.nblocks) return;                      // the whole workgroup leaves together
    const uint64_t r1 = (g.nblocks - r0 < rows_per_wg) ? g.nblocks : r0 + rows_per_wg;
    const uint32_t nrows = (uint32_t)(r1 - r0);
    const uint64_t e0 = r0 * g.inner;
    const uint64_t e1 = (r1 * g.inner < g.n) ? r1 * g.inner : g.n;      // the last block may be short
    const uint64_t j0 = e0 / 4;
    const uint32_t ngroups = (uint32_t)((e1 + 3) / 4 - j0);             // <= kThreads * GPT by the host's choice
    const uint32_t lead = (uint32_t)(e0 - j0 * 4);                      // elements of the first group before the range
    const uint32_t span = (uint32_t)(e1 - e0);
    const uint32_t inner = (uint32_t)g.inner;

    for (uint32_t t = threadIdx.x; t < nrows; t += kThreads) rowmax[t] = 0u;
    __syncthreads();

    uint4 v[GPT];
    uint32_t rows01[GPT], rows23[GPT];       // block of each element relative to r0, 16 bits each (clamped outside the range)
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        if (t < ngroups) v[k] = load_group<VEC>(in, j0 + t, g.n);
    }
    // stochastic rounding: the random words of the first groups are drawn while the loads are in flight
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? (GPT < 4 ? GPT : 4) : 0;
    Words4 early[PRE > 0 ? PRE : 1];
#pragma unroll
    for (int k = 0; k < PRE; ++k) {
        early[k] = random_words(j0 + (threadIdx.x + (uint32_t)k * kThreads), key, 0u);
        asm volatile("" : "+v"(early[k].w[0]), "+v"(early[k].w[1]), "+v"(early[k].w[2]), "+v"(early[k].w[3]));
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        if (t < ngroups) {
            const uint32_t bits[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
            uint32_t mag[4], row[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t at = t * 4u + (uint32_t)e;                  // offset from the first group's start
                const bool mine = at >= lead && at - lead < span;
                const uint32_t off = mine ? at - lead : 0u;
                const uint32_t r = inner == 1u ? off : __umulhi(off, magic);
                row[e] = r < nrows ? r : nrows - 1u;
                mag[e] = mine ? (bits[e] & 0x7fffffffu) : 0u;
            }
            rows01[k] = row[0] | (row[1] << 16);
            rows23[k] = row[2] | (row[3] << 16);
            uint32_t m = mag[0];
#pragma unroll
            for (int e = 1; e < 4; ++e) {
                if (row[e] != row[e - 1]) {
                    atomicMax(&rowmax[row[e - 1]], m);
                    m = 0u;
                }
                m = m > mag[e] ? m : mag[e];
            }
            atomicMax(&rowmax[row[3]], m);
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        if (t < ngroups) {
            const uint64_t j = j0 + t;
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) r = early[k];
            else if (MODE == QSIM_STOCHASTIC) r = random_words(j, key, 0u);
            const uint32_t bits[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
            const uint32_t row[4] = {rows01[k] & 0xffffu, rows01[k] >> 16, rows23[k] & 0xffffu, rows23[k] >> 16};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = quantize_to_grid<MODE>(bits[e], block_plan(rowmax[row[e]], wl, symmetric), r.w[e]);
            const uint32_t at = t * 4u;
            if (at >= lead && at + 3u - lead < span) {
                store_group<VEC>(out, j, g.n, make_uint4(o[0], o[1], o[2], o[3]));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (at + (uint32_t)e >= lead && at + (uint32_t)e - lead < span) out[j * 4 + (uint64_t)e] = o[e];
            }
        }
    }
}

// One contiguous block of up to 16,384 elements per workgroup (outer == 1) when the arrays are not
// aligned or the block length is not a multiple of four: dword accesses; the block is read twice by
// the same workgroup, the second time out of cache.
template <int MODE>
__global__ __launch_bounds__(kThreads) void block_rows_kernel(const uint32_t* in, uint32_t* out, BlockGeom g, int wl,
                                                              int symmetric, RngKey key)
{
    __shared__ uint32_t lds[kThreads / 64];
    const uint64_t b = linear_block();
    if (b >= g.nblocks) return;                       // the whole workgroup leaves together
    const uint64_t start = b * g.inner;
    const uint64_t len = (g.n - start < g.inner) ? g.n - start : g.inner;
    uint32_t m = 0;
    for (uint64_t t = threadIdx.x; t < len; t += kThreads) {
        const uint32_t a = in[start + t] & 0x7fffffffu;
        m = m > a ? m : a;
    }
    const GridPlan p = block_plan(workgroup_max(m, lds), wl, symmetric);
    for (uint64_t t = threadIdx.x; t < len; t += kThreads) {
        const uint64_t i = start + t;
        uint32_t r = 0;
        if (MODE == QSIM_STOCHASTIC) r = random_words(i >> 2, key, 0u).w[i & 3];
        out[i] = quantize_to_grid<MODE>(in[i], p, r);
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
    uint64_t slice_len;    // elements of t per workgroup, a multiple of 4096
    uint32_t slices;       // workgroups per block
};

// Segment number of element t of a block: a 32-bit division whenever the operands allow it (a
// 64-bit one is several times the instructions, and this sits in the inner loops of the general form).
__device__ __forceinline__ uint64_t segment_of(const BlockGeom& g, uint64_t t)
{
    if ((t | g.inner) <= 0xffffffffull) return (uint32_t)t / (uint32_t)g.inner;
    return t / g.inner;
}

__device__ __forceinline__ uint64_t flat_index(const BlockGeom& g, uint64_t b, uint64_t t)
{
    if (g.outer == 1) return b * g.inner + t;
    const uint64_t o = segment_of(g, t), i = t - o * g.inner;
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
    const uint64_t b = linear_block_xz();
    if (b >= sg.g.nblocks) return;                    // the whole workgroup leaves together
    const uint64_t len = block_length(sg, b);
    const uint64_t t0 = (uint64_t)blockIdx.y * sg.slice_len;
    const uint64_t t1 = (t0 + sg.slice_len < len) ? t0 + sg.slice_len : len;
    uint32_t m = 0;
    if (VEC) {
        for (uint64_t t = t0 + 4ull * threadIdx.x; t < t1; t += 4ull * kThreads) {
            const uint64_t i = flat_index(sg.g, b, t);
            uint4 v;
            if (i + 4 <= sg.g.n) v = *reinterpret_cast<const uint4*>(in + i);         // cached: read again in pass 2
            else v = load_group<false>(in, i / 4, sg.g.n);
            const uint32_t gm = max4_mag(v);
            m = m > gm ? m : gm;
        }
    } else {
        // any layout, any alignment: runs of four elements of the block's own numbering; a run that
        // stays inside one segment is one (dword-aligned) dwordx4 access
        for (uint64_t t = t0 + 4ull * threadIdx.x; t < t1; t += 4ull * kThreads) {
            const uint64_t o = sg.g.outer == 1 ? 0 : segment_of(sg.g, t), i = t - o * sg.g.inner;
            if (t + 4 <= t1 && (sg.g.outer == 1 || i + 4 <= sg.g.inner)) {
                const uint64_t at = sg.g.outer == 1 ? b * sg.g.inner + t : (o * sg.g.nblocks + b) * sg.g.inner + i;
                const u32x4 w = *reinterpret_cast<const u32x4_at_dword*>(in + at);       // cached: read again in pass 2
                const uint32_t gm = max4_mag(to_uint4(w));
                m = m > gm ? m : gm;
            } else {
                for (uint64_t e = t; e < t + 4 && e < t1; ++e) {
                    const uint32_t a = in[flat_index(sg.g, b, e)] & 0x7fffffffu;
                    m = m > a ? m : a;
                }
            }
        }
    }
    m = workgroup_max(m, lds);
    if (threadIdx.x == 0) partial[b * sg.slices + blockIdx.y] = m;
}

// Block maxima from the partial maxima of pass 1: block_max[b] = max over s of partial[b * slices + s].
__global__ __launch_bounds__(kThreads) void block_fold_partials_kernel(const uint32_t* partial, uint32_t* block_max,
                                                                       uint64_t nblocks, uint32_t slices)
{
    const uint64_t b = linear_block() * kThreads + threadIdx.x;
    if (b >= nblocks) return;
    uint32_t m = 0;
    for (uint32_t s = 0; s < slices; ++s) {
        const uint32_t a = partial[b * slices + s];
        m = m > a ? m : a;
    }
    block_max[b] = m;
}

// The same with one workgroup per block, for blocks of many slices (one thread would walk them one
// after the other: 512 slices took 33 us).
__global__ __launch_bounds__(kThreads) void block_fold_partials_wide_kernel(const uint32_t* partial, uint32_t* block_max,
                                                                            uint64_t nblocks, uint32_t slices)
{
    __shared__ uint32_t lds[kThreads / 64];
    const uint64_t b = linear_block();
    if (b >= nblocks) return;                          // the whole workgroup leaves together
    uint32_t m = 0;
    for (uint32_t s = threadIdx.x; s < slices; s += kThreads) {
        const uint32_t a = partial[b * slices + s];
        m = m > a ? m : a;
    }
    m = workgroup_max(m, lds);
    if (threadIdx.x == 0) block_max[b] = m;
}

// `npartial` maxima per block are folded: the slices of pass 1, or 1 when the caller supplies
// finished block maxima.
template <int MODE, bool VEC>
__global__ __launch_bounds__(kThreads) void block_apply_kernel(const uint32_t* in, uint32_t* out, const uint32_t* partial,
                                                               uint32_t npartial, SliceGeom sg, int wl, int symmetric,
                                                               RngKey key)
{
    __shared__ uint32_t lds[kThreads / 64];
    const uint64_t b = linear_block_xz();
    if (b >= sg.g.nblocks) return;                    // the whole workgroup leaves together
    uint32_t m = 0;
    for (uint32_t s = threadIdx.x; s < npartial; s += kThreads) {
        const uint32_t a = partial[b * npartial + s];
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
            if (MODE == QSIM_STOCHASTIC) r = random_words(j, key, 0u);
            store_group<true>(out, j, sg.g.n, quantize_group_to_grid<MODE>(v, p, r));
        }
    } else {
        for (uint64_t t = t0 + 4ull * threadIdx.x; t < t1; t += 4ull * kThreads) {
            const uint64_t o = sg.g.outer == 1 ? 0 : segment_of(sg.g, t), i = t - o * sg.g.inner;
            if (t + 4 <= t1 && (sg.g.outer == 1 || i + 4 <= sg.g.inner)) {
                const uint64_t at = sg.g.outer == 1 ? b * sg.g.inner + t : (o * sg.g.nblocks + b) * sg.g.inner + i;
                const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_at_dword*>(in + at));
                Words4 r = {{0u, 0u, 0u, 0u}};
                if (MODE == QSIM_STOCHASTIC) r = random_words_at(at, key, 0u);
                __builtin_nontemporal_store(to_u32x4(quantize_group_to_grid<MODE>(to_uint4(w), p, r)),
                                            reinterpret_cast<u32x4_at_dword*>(out + at));
            } else {
                for (uint64_t e = t; e < t + 4 && e < t1; ++e) {
                    const uint64_t at = flat_index(sg.g, b, e);
                    uint32_t r = 0;
                    if (MODE == QSIM_STOCHASTIC) r = random_words(at >> 2, key, 0u).w[at & 3];
                    out[at] = quantize_to_grid<MODE>(in[at], p, r);
                }
            }
        }
    }
}

// Blocks along an inner dimension (outer > 1) made of short segments: the "column" form, for any
// row length and alignment.  A thread owns a run of four neighbouring columns and a slice of rows
// and walks down its rows, so every access is a coalesced dwordx4 along the row, whatever the
// block length; the block of each of its four columns is fixed, so the index arithmetic (one
// division per column) is paid once per thread.
//   pass 1   per-column maxima of every row slice       -> colmax[slice][column]
//   fold     block maximum = max over slices and over the block's `inner` columns -> blockmax[b]
//   pass 2   the same walk again: quantize with the plans of the four columns' blocks
struct ColumnGeom {
    uint64_t outer;            // rows
    uint32_t row;              // elements per row = nblocks * inner
    uint32_t row_groups;       // runs of four columns per row = ceil(row / 4); colmax rows are 4 * row_groups wide
    uint32_t inner;
    uint32_t nblocks;
    uint32_t slices;           // row slices
    uint32_t rows_per_slice;
};

// A thread's run of four columns in row o starts at element o * row + 4 * c: a group boundary when
// rows are whole groups and the array is aligned (ALIGNED), any dword otherwise.  The last run of a
// row that is not a multiple of four is short and goes element by element.
template <bool ALIGNED>
__device__ __forceinline__ uint4 column_load(const uint32_t* in, uint64_t at, uint32_t have, bool stream)
{
    if (have >= 4u) {
        if (ALIGNED) {
            const u32x4* p = reinterpret_cast<const u32x4*>(in + at);
            return to_uint4(stream ? __builtin_nontemporal_load(p) : *p);
        }
        const u32x4_at_dword* p = reinterpret_cast<const u32x4_at_dword*>(in + at);
        const u32x4 w = stream ? __builtin_nontemporal_load(p) : *p;
        return to_uint4(w);
    }
    uint4 v = {0u, 0u, 0u, 0u};
    if (have > 0u) v.x = in[at];
    if (have > 1u) v.y = in[at + 1];
    if (have > 2u) v.z = in[at + 2];
    return v;
}

template <bool ALIGNED>
__global__ __launch_bounds__(kThreads) void block_column_max_kernel(const uint32_t* in, uint4* colmax, ColumnGeom cg)
{
    const uint32_t c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= cg.row_groups) return;
    const uint64_t o0 = (uint64_t)blockIdx.y * cg.rows_per_slice;
    const uint64_t o1 = (o0 + cg.rows_per_slice < cg.outer) ? o0 + cg.rows_per_slice : cg.outer;
    const uint32_t have = cg.row - 4u * c;                  // columns of this run that exist (4 or more: a whole run)
    uint4 m = {0u, 0u, 0u, 0u};
    for (uint64_t o = o0; o < o1; o += 4) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[k] = make_uint4(0u, 0u, 0u, 0u);
            if (o + k < o1) v[k] = column_load<ALIGNED>(in, (o + k) * cg.row + 4ull * c, have, false);   // cached: read again in pass 2
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t a0 = v[k].x & 0x7fffffffu, a1 = v[k].y & 0x7fffffffu;
            const uint32_t a2 = v[k].z & 0x7fffffffu, a3 = v[k].w & 0x7fffffffu;
            m.x = m.x > a0 ? m.x : a0;
            m.y = m.y > a1 ? m.y : a1;
            m.z = m.z > a2 ? m.z : a2;
            m.w = m.w > a3 ? m.w : a3;
        }
    }
    colmax[(uint64_t)blockIdx.y * cg.row_groups + c] = m;
}

// One wavefront per block: lanes stride over the block's slices * inner column maxima.
__global__ __launch_bounds__(kThreads) void block_column_fold_kernel(const uint32_t* colmax, uint32_t* blockmax, ColumnGeom cg)
{
    const uint64_t b = linear_block() * (kThreads / 64) + (threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63;
    uint32_t m = 0;
    if (b < cg.nblocks) {
        const uint64_t row = 4ull * cg.row_groups;
        const uint32_t count = cg.slices * cg.inner;
        for (uint32_t t = lane; t < count; t += 64) {
            const uint32_t s = t / cg.inner, i = t - s * cg.inner;
            const uint32_t a = colmax[s * row + b * cg.inner + i];
            m = m > a ? m : a;
        }
    }
    m = wave_max(m);
    if (lane == 0 && b < cg.nblocks) blockmax[b] = m;
}

// The same fold with one THREAD per block, for blocks of few columns and few slices (a wavefront
// per block would leave most of its lanes idle and need millions of workgroups).
__global__ __launch_bounds__(kThreads) void block_column_fold_small_kernel(const uint32_t* colmax, uint32_t* blockmax, ColumnGeom cg)
{
    const uint64_t b = linear_block() * kThreads + threadIdx.x;
    if (b >= cg.nblocks) return;
    uint32_t m = 0;
    for (uint32_t s = 0; s < cg.slices; ++s) {
        const uint32_t* p = colmax + (uint64_t)s * (4ull * cg.row_groups) + b * cg.inner;
        for (uint32_t i = 0; i < cg.inner; ++i) m = m > p[i] ? m : p[i];
    }
    blockmax[b] = m;
}

template <int MODE, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void block_column_apply_kernel(const uint32_t* in, uint32_t* out,
                                                                      const uint32_t* blockmax, ColumnGeom cg, int wl,
                                                                      int symmetric, RngKey key)
{
    const uint32_t c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= cg.row_groups) return;
    const uint64_t o0 = (uint64_t)blockIdx.y * cg.rows_per_slice;
    const uint64_t o1 = (o0 + cg.rows_per_slice < cg.outer) ? o0 + cg.rows_per_slice : cg.outer;
    const uint32_t have = cg.row - 4u * c;
    GridPlan p[4];
    if (cg.inner % 4 == 0) {
        p[0] = p[1] = p[2] = p[3] = block_plan(blockmax[(4u * c) / cg.inner], wl, symmetric);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t col = 4u * c + (uint32_t)e < cg.row ? 4u * c + (uint32_t)e : cg.row - 1u;
            p[e] = block_plan(blockmax[col / cg.inner], wl, symmetric);
        }
    }
    for (uint64_t o = o0; o < o1; o += 4) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (o + k < o1) v[k] = column_load<ALIGNED>(in, (o + k) * cg.row + 4ull * c, have, true);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (o + k < o1) {
                const uint64_t at = (o + k) * cg.row + 4ull * c;
                Words4 r = {{0u, 0u, 0u, 0u}};
                if (MODE == QSIM_STOCHASTIC) r = ALIGNED ? random_words(at >> 2, key, 0u) : random_words_at(at, key, 0u);
                uint4 q;
                q.x = quantize_to_grid<MODE>(v[k].x, p[0], r.w[0]);
                q.y = quantize_to_grid<MODE>(v[k].y, p[1], r.w[1]);
                q.z = quantize_to_grid<MODE>(v[k].z, p[2], r.w[2]);
                q.w = quantize_to_grid<MODE>(v[k].w, p[3], r.w[3]);
                if (have >= 4u) {
                    if (ALIGNED) __builtin_nontemporal_store(to_u32x4(q), reinterpret_cast<u32x4*>(out + at));
                    else __builtin_nontemporal_store(to_u32x4(q), reinterpret_cast<u32x4_at_dword*>(out + at));
                } else {
                    if (have > 0u) out[at] = q.x;
                    if (have > 1u) out[at + 1] = q.y;
                    if (have > 2u) out[at + 2] = q.z;
                }
            }
        }
    }
}

// Blocks along an inner dimension (outer > 1) with SHORT rows (nblocks * inner <= 61,440 elements,
// nblocks <= 4096), any inner, any alignment: the "flat" form.  The tensor is walked in its own
// groups of four, front to back, by a fixed number of workgroups that each own one contiguous
// range; the block of an element follows from its position in the row,
//     b = ((first position of the step + offset) mod row) div inner,
// both by one multiply-high with a host-made reciprocal (exact below 2^16).  Block maxima are
// collected in an LDS table per workgroup (ds_max), written out as partial[workgroup][block]
// (no atomics in memory, nothing to initialise), folded by block_fold_rows_kernel in two steps,
// and pass 2 walks the same ranges with the finished maxima in LDS.
constexpr int kFlatMaxBlocks = 4096;
constexpr uint32_t kFlatMaxRow = 61440;                   // row + one step of 4096 elements stays below 2^16
constexpr int kFlatGpt = 4;                               // groups per thread and step
constexpr uint32_t kFlatStepGroups = kThreads * kFlatGpt;   // 4096 elements per step

struct FlatGeom {
    uint64_t n, groups;          // elements, groups of four
    uint64_t groups_per_wg;      // a multiple of kFlatStepGroups
    uint32_t row, inner, nblocks;
    uint32_t magic_row, magic_inner;   // floor(2^32 / d) + 1 (unused when d == 1)
    uint32_t wgs;
    uint32_t copies;             // copies of the LDS table in pass 1: a power of two, 1..64, copies * nblocks <= 4096
};

__device__ __forceinline__ uint32_t flat_block(const FlatGeom& fg, uint32_t pos /* < 2^16 */)
{
    const uint32_t in_row = fg.row == 1u ? 0u : pos - __umulhi(pos, fg.magic_row) * fg.row;
    return fg.inner == 1u ? in_row : __umulhi(in_row, fg.magic_inner);
}

// The groups of one step.  A step that lies wholly inside the array (all but the last) issues its
// loads back to back with nothing in between, so that all of them are in flight together.
__device__ __forceinline__ void flat_load_step(const uint32_t* in, uint64_t base, const FlatGeom& fg, uint4 (&v)[kFlatGpt])
{
    if ((base + kFlatStepGroups) * 4 <= fg.n) {                              // wave-uniform
        const u32x4_at_dword* p = reinterpret_cast<const u32x4_at_dword*>(in + base * 4) + threadIdx.x;
#pragma unroll
        for (int k = 0; k < kFlatGpt; ++k) {
            const u32x4 w = __builtin_nontemporal_load(p + k * kThreads);
            v[k] = to_uint4(w);
        }
    } else {
#pragma unroll
        for (int k = 0; k < kFlatGpt; ++k) {
            const uint64_t j = base + threadIdx.x + (uint64_t)k * kThreads;
            v[k] = make_uint4(0u, 0u, 0u, 0u);
            if (j < fg.groups) v[k] = load_group<false>(in, j, fg.n);
        }
    }
}

__global__ __launch_bounds__(kThreads) void block_flat_max_kernel(const uint32_t* in, uint32_t* partial, FlatGeom fg)
{
    // Few blocks mean many lanes per block, and same-address LDS atomics of one instruction are
    // carried out one after the other: so the table is replicated, lane l works on copy l mod copies
    // (copies * nblocks <= 4096), and the copies are folded at the end.
    __shared__ uint32_t table[kFlatMaxBlocks];
    const uint32_t copies = fg.copies;
    for (uint32_t t = threadIdx.x; t < fg.nblocks * copies; t += kThreads) table[t] = 0u;
    __syncthreads();
    uint32_t* mine = table + (threadIdx.x & (copies - 1u)) * fg.nblocks;
    // steps are dealt out round-robin, so that at any moment the workgroups together read one
    // contiguous front of the tensor
    const uint64_t g1 = fg.groups;
    for (uint64_t base = (uint64_t)blockIdx.x * kFlatStepGroups; base < g1; base += (uint64_t)fg.wgs * kFlatStepGroups) {
        const uint32_t pos0 = (uint32_t)((base * 4) % fg.row);            // wave-uniform
        uint4 v[kFlatGpt];
        flat_load_step(in, base, fg, v);
#pragma unroll
        for (int k = 0; k < kFlatGpt; ++k) {
            const uint64_t j = base + threadIdx.x + (uint64_t)k * kThreads;
            if (j < g1) {
                const uint32_t off = (threadIdx.x + (uint32_t)k * kThreads) * 4u;
                if (fg.inner % 4u == 0u) {                                    // a group never straddles blocks
                    atomicMax(&mine[flat_block(fg, pos0 + off)], max4_mag(v[k]));
                } else {
                    const uint32_t mag[4] = {v[k].x & 0x7fffffffu, v[k].y & 0x7fffffffu, v[k].z & 0x7fffffffu,
                                             v[k].w & 0x7fffffffu};
                    uint32_t prev = flat_block(fg, pos0 + off), m = mag[0];
#pragma unroll
                    for (uint32_t e = 1; e < 4; ++e) {
                        // elements past the end read as zero; their block number is still a valid one
                        const uint32_t b = flat_block(fg, pos0 + off + e);
                        if (b != prev) {
                            atomicMax(&mine[prev], m);
                            m = 0u;
                            prev = b;
                        }
                        m = m > mag[e] ? m : mag[e];
                    }
                    atomicMax(&mine[prev], m);
                }
            }
        }
    }
    __syncthreads();
    for (uint32_t t = threadIdx.x; t < fg.nblocks; t += kThreads) {
        uint32_t m = table[t];
        for (uint32_t c = 1; c < copies; ++c) {
            const uint32_t a = table[c * fg.nblocks + t];
            m = m > a ? m : a;
        }
        partial[(uint64_t)blockIdx.x * fg.nblocks + t] = m;
    }
}

// dst[p * nblocks + b] = max over the rows k of part p of src[k * nblocks + b]; `rows` rows are cut
// into `parts` parts.  One thread per (p, b): neighbouring threads read neighbouring blocks.
__global__ __launch_bounds__(kThreads) void block_fold_rows_kernel(const uint32_t* src, uint32_t* dst, uint32_t nblocks,
                                                                   uint32_t rows, uint32_t parts)
{
    const uint32_t b = blockIdx.x * kThreads + threadIdx.x;
    const uint32_t p = blockIdx.y;
    if (b >= nblocks) return;
    const uint32_t per = (rows + parts - 1) / parts;
    const uint32_t k0 = p * per;
    const uint32_t k1 = (k0 + per < rows) ? k0 + per : rows;
    uint32_t m = 0;
#pragma unroll 8
    for (uint32_t k = k0; k < k1; ++k) {
        const uint32_t a = src[(uint64_t)k * nblocks + b];
        m = m > a ? m : a;
    }
    dst[(uint64_t)p * nblocks + b] = m;
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void block_flat_apply_kernel(const uint32_t* in, uint32_t* out, const uint32_t* blockmax,
                                                                    FlatGeom fg, int wl, int symmetric, RngKey key)
{
    __shared__ uint32_t table[kFlatMaxBlocks];
    for (uint32_t t = threadIdx.x; t < fg.nblocks; t += kThreads) table[t] = blockmax[t];
    __syncthreads();
    // steps are dealt out round-robin, so that at any moment the workgroups together read one
    // contiguous front of the tensor
    const uint64_t g1 = fg.groups;
    for (uint64_t base = (uint64_t)blockIdx.x * kFlatStepGroups; base < g1; base += (uint64_t)fg.wgs * kFlatStepGroups) {
        const uint32_t pos0 = (uint32_t)((base * 4) % fg.row);            // wave-uniform
        uint4 v[kFlatGpt];
        flat_load_step(in, base, fg, v);
#pragma unroll
        for (int k = 0; k < kFlatGpt; ++k) {
            const uint64_t j = base + threadIdx.x + (uint64_t)k * kThreads;
            if (j < g1) {
                const uint32_t off = (threadIdx.x + (uint32_t)k * kThreads) * 4u;
                Words4 r = {{0u, 0u, 0u, 0u}};
                if (MODE == QSIM_STOCHASTIC) r = random_words(j, key, 0u);
                uint4 o;
                if (fg.inner % 4u == 0u) {
                    o = quantize_group_to_grid<MODE>(v[k], block_plan(table[flat_block(fg, pos0 + off)], wl, symmetric), r);
                } else {
                    o.x = quantize_to_grid<MODE>(v[k].x, block_plan(table[flat_block(fg, pos0 + off)], wl, symmetric), r.w[0]);
                    o.y = quantize_to_grid<MODE>(v[k].y, block_plan(table[flat_block(fg, pos0 + off + 1u)], wl, symmetric), r.w[1]);
                    o.z = quantize_to_grid<MODE>(v[k].z, block_plan(table[flat_block(fg, pos0 + off + 2u)], wl, symmetric), r.w[2]);
                    o.w = quantize_to_grid<MODE>(v[k].w, block_plan(table[flat_block(fg, pos0 + off + 3u)], wl, symmetric), r.w[3]);
                }
                store_group<false>(out, j, fg.n, o);
            }
        }
    }
}

// Contiguous blocks spread over several workgroups (outer == 1, inner % 4 == 0, aligned arrays):
// the streaming forms of the two passes.  Workgroup (s, b) owns slice s of block b in both passes
// and walks it in steps of 4096 elements with four loads in flight per thread.  Pass 1 writes the
// slice's maximum to partial[b * slices + s]; pass 2 folds the partials of its block once, then
// quantizes its slice.
constexpr int kTileGroups = 4 * kThreads;          // groups per workgroup step: 4096 elements

struct SliceView {
    uint64_t end;      // one past the last element of the block (flat index)
    uint64_t j0;       // first group of the slice
    uint64_t groups;   // groups in the slice
};

__device__ __forceinline__ SliceView slice_view(const SliceGeom& sg, uint64_t b, uint64_t s)
{
    const uint64_t start = b * sg.g.inner;
    const uint64_t len = block_length(sg, b);
    const uint64_t t0 = s * sg.slice_len;
    const uint64_t t1 = (t0 + sg.slice_len < len) ? t0 + sg.slice_len : len;
    SliceView v;
    v.end = start + len;
    v.j0 = (start + t0) / 4;
    v.groups = t1 > t0 ? (t1 - t0 + 3) / 4 : 0;
    return v;
}

// Largest magnitude encoding of a slice, read with plain (cached) loads.
__device__ __forceinline__ uint32_t slice_max(const uint32_t* in, const SliceView& sv)
{
    uint32_t m = 0;
    for (uint64_t base = threadIdx.x; base < sv.groups; base += kTileGroups) {
        uint4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint64_t t = base + (uint64_t)k * kThreads;
            v[k] = make_uint4(0u, 0u, 0u, 0u);
            if (t < sv.groups) {
                const uint64_t i = (sv.j0 + t) * 4;
                if (i + 4 <= sv.end) v[k] = *reinterpret_cast<const uint4*>(in + i);
                else v[k] = load_group<false>(in, sv.j0 + t, sv.end);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t gm = max4_mag(v[k]);
            m = m > gm ? m : gm;
        }
    }
    return m;
}

__global__ __launch_bounds__(kThreads) void block_slice_max_kernel(const uint32_t* in, uint32_t* partial, SliceGeom sg)
{
    __shared__ uint32_t lds[kThreads / 64];
    for (uint64_t b = blockIdx.y; b < sg.g.nblocks; b += gridDim.y) {
        const uint32_t m = workgroup_max(slice_max(in, slice_view(sg, b, blockIdx.x)), lds);
        if (threadIdx.x == 0) partial[b * sg.slices + blockIdx.x] = m;
    }
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void block_slice_apply_kernel(const uint32_t* in, uint32_t* out,
                                                                     const uint32_t* partial, uint32_t npartial, SliceGeom sg,
                                                                     int wl, int symmetric, RngKey key)
{
    // `npartial` maxima per block are folded: the slices of pass 1, or 1 when the caller supplies finished maxima
    __shared__ uint32_t lds[kThreads / 64];
    for (uint64_t b = blockIdx.y; b < sg.g.nblocks; b += gridDim.y) {
        uint32_t m = 0;
        for (uint32_t s = threadIdx.x; s < npartial; s += kThreads) {
            const uint32_t a = partial[b * npartial + s];
            m = m > a ? m : a;
        }
        const GridPlan p = block_plan(workgroup_max(m, lds), wl, symmetric);
        const SliceView sv = slice_view(sg, b, blockIdx.x);
        for (uint64_t base = threadIdx.x; base < sv.groups; base += kTileGroups) {
            uint4 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint64_t t = base + (uint64_t)k * kThreads;
                if (t < sv.groups) v[k] = load_group<true>(in, sv.j0 + t, sv.end);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint64_t t = base + (uint64_t)k * kThreads;
                if (t < sv.groups) {
                    Words4 r = {{0u, 0u, 0u, 0u}};
                    if (MODE == QSIM_STOCHASTIC) r = random_words(sv.j0 + t, key, 0u);
                    store_group<true>(out, sv.j0 + t, sv.end, quantize_group_to_grid<MODE>(v[k], p, r));
                }
            }
        }
    }
}

// Single pass for contiguous blocks that fit in the register files of the whole chip (for instance
// a 4096 x 4096 tensor quantized as one block).  The grid is small enough for every workgroup to be
// resident at the same time; each loads its slice of 256 * GPT groups into registers, publishes the
// slice's maximum, waits until all workgroups have arrived, folds the maxima of its block and
// quantizes out of registers: HBM sees each element once in and once out.
//
// Scratch layout (zeroed by block_sync_clear_kernel before the launch; every counter and flag has
// a 64-byte line to itself):
//   sync[0]                              arrivals of whole groups of 32 workgroups
//   sync[16 * (1 + c)],   c < 32         "everyone has arrived" flag, 32 copies
//   sync[16 * (33 + g)],  g < 128        arrivals inside group g = workgroup / 32
//   sync[kSyncSlots0 + w]                slot of workgroup w: its maximum with the top bit set as a
//                                        "published" mark (magnitude encodings have that bit clear)
// Arrival is two-level and the wait polls one of 32 flag copies, so no address sees more than a
// few dozen device-scope operations: a single counter polled by a thousand workgroups serialises
// at its memory channel and costs far more than the kernel's whole memory traffic.
//
// The wait is bounded in time.  A workgroup whose wait runs out (the device is shared with other
// work, so not every workgroup got a slot) still produces the right result: for every slot of its block that is not yet published
// it computes the slice's maximum from memory itself.  That is safe even in place, because a
// workgroup writes its output only after its own wait, which starts after it has published; so if
// the slot is still unpublished after the read, the read saw nothing but input.
constexpr uint32_t kSyncFlagCopies = 32;
constexpr uint32_t kSyncGroup = 32;                // workgroups per first-level counter
constexpr uint32_t kSyncMaxGroups = 128;
constexpr uint32_t kSyncSlots0 = 16 * (1 + kSyncFlagCopies + kSyncMaxGroups);
constexpr uint32_t kPublished = 0x80000000u;

__global__ void block_sync_clear_kernel(uint32_t* sync, uint32_t words)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < words) sync[i] = 0u;
}

struct ResidentGeom {
    SliceGeom sg;            // slice_len = 1024 * GPT elements; slices = workgroups per block
    uint32_t total_wgs;      // nblocks * slices
    uint32_t wait_us;        // microseconds a workgroup waits for the others before the fallback
};

// With 16 groups per thread the kernel must keep to 128 VGPRs (four waves per SIMD, four workgroups
// per CU): that is what lets 1024 workgroups hold a 16 Mi-element tensor.
//
// CLUSTER: the tensor as a whole does not fit, but each block does (at most 64 slices), and the
// grid may be far larger than the chip.  Only the workgroups of one block meet: each publishes its
// slot and polls the slots of its block (one lane per slot) instead of the counters and flags.
// Workgroups are numbered block by block and dispatched in that order, so the workgroups of the
// lowest unfinished block are always among the resident ones and the grid drains block after
// block; should the dispatcher ever do otherwise, the bounded wait and the exact fallback below
// still end every workgroup with the right result.
template <int MODE, int GPT, bool CLUSTER = false>
__global__ __launch_bounds__(kThreads, (GPT >= 16 ? 4 : 1)) void block_resident_kernel(const uint32_t* in, uint32_t* out, uint32_t* sync,
                                                                  ResidentGeom rg, int wl, int symmetric, RngKey key)
{
    // Stochastic rounding: the random words of the first PRE groups are drawn while the loads are
    // in flight and parked in LDS (36 KiB at most, so four workgroups still share a CU); after the
    // wait only the remaining groups pay for Philox, and the arithmetic hides behind the stores.
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? (GPT < 9 ? GPT : 9) : 0;
    __shared__ uint4 parked[PRE > 0 ? PRE * kThreads : 1];
    __shared__ uint32_t lds[kThreads / 64];
    __shared__ uint32_t shared_word;
    const uint32_t wg = CLUSTER ? (uint32_t)linear_block() : blockIdx.x;
    if (CLUSTER && wg >= rg.total_wgs) return;                   // the whole workgroup leaves together
    const uint32_t b = wg / rg.sg.slices, s = wg - b * rg.sg.slices;
    const SliceView sv = slice_view(rg.sg, b, s);
    uint32_t* slots = sync + kSyncSlots0;

    // the slice is addressed from a wave-uniform base with small per-thread offsets, which keeps
    // the address arithmetic out of the vector registers that hold the data
    const uint32_t* sin = in + sv.j0 * 4;
    uint32_t* sout = out + sv.j0 * 4;
    const uint64_t slice_end = sv.end - sv.j0 * 4;               // elements reachable from the base
    const int ngroups = (int)sv.groups;
    const bool full = ngroups == kThreads * GPT && slice_end >= 4ull * kThreads * GPT;

    uint4 v[GPT];
    uint32_t m = 0;
    if (full) {
#pragma unroll
        for (int k = 0; k < GPT; ++k) {
            const int t = (int)threadIdx.x + k * kThreads;
            v[k] = to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(sin) + t));
        }
    } else {
#pragma unroll
        for (int k = 0; k < GPT; ++k) {
            const int t = (int)threadIdx.x + k * kThreads;
            v[k] = make_uint4(0u, 0u, 0u, 0u);
            if (t < ngroups) v[k] = load_group<true>(sin, (uint64_t)t, slice_end);
        }
    }
#pragma unroll
    for (int k = 0; k < PRE; ++k) {
        const Words4 r = random_words(sv.j0 + (uint64_t)((int)threadIdx.x + k * kThreads), key, 0u);
        parked[k * kThreads + threadIdx.x] = make_uint4(r.w[0], r.w[1], r.w[2], r.w[3]);
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t gm = max4_mag(v[k]);
        m = m > gm ? m : gm;
    }
    m = workgroup_max(m, lds);

    // All communication is through relaxed device-scope atomics on words that only atomics touch:
    // nothing else has to become visible between workgroups, so no release or acquire fence (each
    // of which writes back or invalidates a whole L2 on this multi-die part) is needed.  Order is
    // kept by waiting for the returned value of one atomic before the next one is issued.
    if (CLUSTER) {
        if (threadIdx.x == 0) {
            uint32_t old = __hip_atomic_exchange(&slots[wg], m | kPublished, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(old) : : "memory");
        }
        if (threadIdx.x < 64) {
            // the first wavefront polls: lane i watches slot i of the block (slices <= 64)
            const uint32_t* watched = slots + (uint64_t)b * rg.sg.slices + (threadIdx.x < rg.sg.slices ? threadIdx.x : 0u);
            const uint64_t t0 = __builtin_amdgcn_s_memrealtime();        // 100 MHz
            const uint64_t budget = (uint64_t)rg.wait_us * 100u;
            bool all = __all((__hip_atomic_load(watched, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kPublished) != 0u);
            while (!all && __builtin_amdgcn_s_memrealtime() - t0 < budget) {
                __builtin_amdgcn_s_sleep(2);
                all = __all((__hip_atomic_load(watched, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kPublished) != 0u);
            }
            if (threadIdx.x == 0) shared_word = all ? 1u : 0u;
        }
    } else if (threadIdx.x == 0) {
        uint32_t old = __hip_atomic_exchange(&slots[wg], m | kPublished, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(old) : : "memory");       // the slot is published before we count
        const uint32_t group = wg / kSyncGroup;
        const uint32_t ngroups_sync = (rg.total_wgs + kSyncGroup - 1) / kSyncGroup;
        const uint32_t in_group = (group + 1 == ngroups_sync) ? rg.total_wgs - group * kSyncGroup : kSyncGroup;
        uint32_t* flags = sync + 16;
        if (__hip_atomic_fetch_add(&sync[16 * (1 + kSyncFlagCopies + group)], 1u, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT) == in_group - 1u) {
            if (__hip_atomic_fetch_add(&sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == ngroups_sync - 1u) {
                for (uint32_t c = 0; c < kSyncFlagCopies; ++c)
                    __hip_atomic_store(&flags[16 * c], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        const uint32_t* my_flag = &flags[16 * (wg % kSyncFlagCopies)];
        const uint64_t t0 = __builtin_amdgcn_s_memrealtime();            // 100 MHz
        const uint64_t budget = (uint64_t)rg.wait_us * 100u;
        bool all = __hip_atomic_load(my_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
        while (!all && __builtin_amdgcn_s_memrealtime() - t0 < budget) {
            __builtin_amdgcn_s_sleep(2);
            all = __hip_atomic_load(my_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
        }
        shared_word = all ? 1u : 0u;
    }
    __syncthreads();
    const bool all_arrived = shared_word != 0u;

    uint32_t bm = 0;
    uint32_t* mine = slots + (uint64_t)b * rg.sg.slices;
    if (all_arrived) {
        for (uint32_t i = threadIdx.x; i < rg.sg.slices; i += kThreads) {
            const uint32_t a = __hip_atomic_load(&mine[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & ~kPublished;
            bm = bm > a ? bm : a;
        }
        bm = workgroup_max(bm, lds);
    } else {
        for (uint32_t i = 0; i < rg.sg.slices; ++i) {
            __syncthreads();
            if (threadIdx.x == 0) shared_word = __hip_atomic_load(&mine[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            uint32_t a = shared_word;
            if (!(a & kPublished)) {
                // the owner of slice i has not published, so it has not written any output yet:
                // read its input; if the slot is still unpublished afterwards, the read was clean
                const uint32_t own = workgroup_max(slice_max(in, slice_view(rg.sg, b, i)), lds);
                __syncthreads();
                if (threadIdx.x == 0) shared_word = __hip_atomic_load(&mine[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __syncthreads();
                a = (shared_word & kPublished) ? shared_word : own;
            }
            a &= ~kPublished;
            bm = bm > a ? bm : a;
        }
    }

    const GridPlan p = block_plan(bm, wl, symmetric);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const int t = (int)threadIdx.x + k * kThreads;
        if (full || t < ngroups) {
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) {
                const uint4 w = parked[k * kThreads + threadIdx.x];
                r = Words4{{w.x, w.y, w.z, w.w}};
            } else if (MODE == QSIM_STOCHASTIC) {
                r = random_words(sv.j0 + (uint64_t)t, key, 0u);
            }
            const uint4 o = quantize_group_to_grid<MODE>(v[k], p, r);
            if (full) __builtin_nontemporal_store(to_u32x4(o), reinterpret_cast<u32x4*>(sout) + t);
            else store_group<true>(sout, (uint64_t)t, slice_end, o);
        }
    }
}

// The meeting of the workgroups of one block, as in the kernel above: workgroup s publishes its
// maximum m in slot s of the block's `slices` slots (zeroed before the launch) and gets the block's
// maximum back.  The first wavefront polls, every lane up to slices / 64 slots, for at most wait_us;
// when that runs out, every slot still unpublished is recomputed from memory with
// slice_max(i), each thread's share of the maximum of slice i (safe for the reason given above).
// Called by every thread of the workgroup.
template <class SliceMax>
__device__ __forceinline__ uint32_t meet_in_block(uint32_t* mine, uint32_t s, uint32_t slices, uint32_t m, uint32_t wait_us,
                                                  uint32_t* lds, uint32_t& shared_word, SliceMax slice_max)
{
    // relaxed device-scope atomics on words only atomics touch; order by waiting for returned values
    if (threadIdx.x == 0) {
        uint32_t old = __hip_atomic_exchange(&mine[s], m | kPublished, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(old) : : "memory");
    }
    if (threadIdx.x < 64) {
        const uint64_t start = __builtin_amdgcn_s_memrealtime();     // 100 MHz
        const uint64_t budget = (uint64_t)wait_us * 100u;
        bool all;
        for (;;) {
            bool ok = true;
            for (uint32_t i = threadIdx.x; i < slices; i += 64u)
                ok = ok && (__hip_atomic_load(&mine[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kPublished) != 0u;
            all = __all(ok);
            if (all || __builtin_amdgcn_s_memrealtime() - start >= budget) break;
            __builtin_amdgcn_s_sleep(2);
        }
        if (threadIdx.x == 0) shared_word = all ? 1u : 0u;
    }
    __syncthreads();
    const bool all_arrived = shared_word != 0u;

    uint32_t bm = 0;
    if (all_arrived) {
        for (uint32_t i = threadIdx.x; i < slices; i += kThreads) {
            const uint32_t a = __hip_atomic_load(&mine[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & ~kPublished;
            bm = bm > a ? bm : a;
        }
        return workgroup_max(bm, lds);
    }
    for (uint32_t i = 0; i < slices; ++i) {
        __syncthreads();
        if (threadIdx.x == 0) shared_word = __hip_atomic_load(&mine[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        uint32_t a = shared_word;
        if (!(a & kPublished)) {
            // the owner of slice i has not published, so it has not written any output yet:
            // read its input; if the slot is still unpublished afterwards, the read was clean
            const uint32_t own = workgroup_max(slice_max(i), lds);
            __syncthreads();
            if (threadIdx.x == 0) shared_word = __hip_atomic_load(&mine[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            a = (shared_word & kPublished) ? shared_word : own;
        }
        a &= ~kPublished;
        bm = bm > a ? bm : a;
    }
    return bm;
}

// The same block-by-block single pass for blocks along an inner dimension (outer > 1) made of
// aligned segments of at least 64 elements (inner % 4 == 0): per-channel blocks of an
// [N, C, H, W] tensor.  Slice s of block b is elements [s * 16384, ...) of the block's own
// numbering t = o * inner + i; a group's place in the array follows from one division by `inner`
// (multiply-high with a reciprocal rounded up, corrected by at most one).  Up to 256 slices per
// block; every lane of the polling wavefront watches up to four slots.  `slots`: one word per
// workgroup, zeroed before the launch.
constexpr uint32_t kStridedSliceLen = 4u * kThreads * 16u;
constexpr uint32_t kStridedMaxSlices = 256;

struct StridedClusterGeom {
    uint64_t nblocks;
    uint32_t block_len;      // outer * inner, at most kStridedMaxSlices * kStridedSliceLen
    uint32_t slices;
    uint32_t inner;          // a multiple of 4, at least 64
    uint32_t magic_inner;    // floor(2^32 / inner) + 1
    uint32_t total_wgs;
    uint32_t wait_us;
};

// Group number, in the array, of the group at element tt (a multiple of 4) of block b.
__device__ __forceinline__ uint64_t strided_group(const StridedClusterGeom& cg, uint32_t b, uint32_t tt)
{
    uint32_t o = __umulhi(tt, cg.magic_inner);           // tt / inner or one more (tt < 2^22)
    uint32_t i = tt - o * cg.inner;
    if ((int32_t)i < 0) {
        o -= 1u;
        i += cg.inner;
    }
    return (((uint64_t)o * cg.nblocks + b) * cg.inner + i) >> 2;
}

__device__ __forceinline__ uint32_t strided_slice_groups(const StridedClusterGeom& cg, uint32_t s)
{
    const uint32_t t0 = s * kStridedSliceLen;
    const uint32_t t1 = (cg.block_len - t0 < kStridedSliceLen) ? cg.block_len : t0 + kStridedSliceLen;
    return (t1 - t0) / 4u;
}

template <int MODE>
__global__ __launch_bounds__(kThreads, 4) void block_cluster_strided_kernel(const uint32_t* in, uint32_t* out, uint32_t* slots,
                                                                            StridedClusterGeom cg, int wl, int symmetric,
                                                                            RngKey key)
{
    constexpr int GPT = 16;
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? 9 : 0;          // random words parked in LDS, as in the kernel above
    __shared__ uint4 parked[PRE > 0 ? PRE * kThreads : 1];
    __shared__ uint32_t lds[kThreads / 64];
    __shared__ uint32_t shared_word;
    const uint32_t wg = (uint32_t)linear_block();
    if (wg >= cg.total_wgs) return;                                // the whole workgroup leaves together
    const uint32_t b = wg / cg.slices, s = wg - b * cg.slices;
    const uint32_t t0 = s * kStridedSliceLen;
    const uint32_t ngroups = strided_slice_groups(cg, s);

    uint4 v[GPT];
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        if (t < ngroups) {
            const uint64_t j = strided_group(cg, b, t0 + 4u * t);
            v[k] = to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(in) + j));
            if (k < PRE) {
                const Words4 r = random_words(j, key, 0u);
                parked[k * kThreads + threadIdx.x] = make_uint4(r.w[0], r.w[1], r.w[2], r.w[3]);
            }
        }
    }
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t gm = max4_mag(v[k]);
        m = m > gm ? m : gm;
    }
    m = workgroup_max(m, lds);

    uint32_t* mine = slots + (uint64_t)b * cg.slices;
    const uint32_t bm = meet_in_block(mine, s, cg.slices, m, cg.wait_us, lds, shared_word, [&](uint32_t i) {
        uint32_t own = 0;
        const uint32_t count = strided_slice_groups(cg, i);
        for (uint32_t t = threadIdx.x; t < count; t += kThreads) {
            const uint4 w = *(reinterpret_cast<const uint4*>(in) + strided_group(cg, b, i * kStridedSliceLen + 4u * t));
            const uint32_t gm = max4_mag(w);
            own = own > gm ? own : gm;
        }
        return own;
    });

    const GridPlan p = block_plan(bm, wl, symmetric);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        if (t < ngroups) {
            const uint64_t j = strided_group(cg, b, t0 + 4u * t);
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) {
                const uint4 w = parked[k * kThreads + threadIdx.x];
                r = Words4{{w.x, w.y, w.z, w.w}};
            } else if (MODE == QSIM_STOCHASTIC) {
                r = random_words(j, key, 0u);
            }
            __builtin_nontemporal_store(to_u32x4(quantize_group_to_grid<MODE>(v[k], p, r)), reinterpret_cast<u32x4*>(out) + j);
        }
    }
}

// The same for segments of any length from 64 elements at any alignment (inner % 4 != 0, or arrays
// that are only dword aligned): per-channel blocks of an [N, C, 27, 27] tensor.  The unit is still
// a group of the ARRAY's numbering (elements 4j .. 4j + 3), so that one Philox block serves it;
// a segment starting at element S is covered by groups S / 4 ... (S + inner - 1) / 4, of which the
// first and the last may hold elements of a neighbouring block ("strangers": loaded, because one
// dwordx4 load at a dword-aligned address is still the cheapest, then masked out of the maximum and
// never stored).  Every segment is given G = (inner + 2) / 4 + 1 group slots, the most it can
// cover; slot t of a block is slot u = t % G of segment o = t / G, unused when that segment covers
// fewer groups.  The slots of a block are dealt out evenly to its slices, at most 4096 each.
struct RaggedClusterGeom {
    uint64_t n;
    uint64_t nblocks;
    uint32_t inner;          // at least 64
    uint32_t seg_groups;     // G
    uint32_t magic_groups;   // floor(2^32 / G) + 1
    uint32_t block_groups;   // outer * G, at most kStridedMaxSlices * 4096
    uint32_t slices;         // ceil(block_groups / 4096)
    uint32_t slice_groups;   // ceil(block_groups / slices): the slots are dealt out evenly
    uint32_t total_wgs;
    uint32_t wait_us;
};

constexpr uint32_t kRaggedSliceGroups = kThreads * 16u;

// Slot t of block b: the group j it stands for and which of its four elements belong to the block
// (bit e of `mask`; 0 for an unused slot).
__device__ __forceinline__ void ragged_slot(const RaggedClusterGeom& cg, uint32_t b, uint32_t t, uint64_t& j, uint32_t& mask)
{
    uint32_t o = __umulhi(t, cg.magic_groups);            // t / G or one more (t < 2^20)
    uint32_t u = t - o * cg.seg_groups;
    if ((int32_t)u < 0) {
        o -= 1u;
        u += cg.seg_groups;
    }
    const uint64_t start = ((uint64_t)o * cg.nblocks + b) * cg.inner;      // first element of the segment
    const uint32_t r = (uint32_t)start & 3u;
    j = (start >> 2) + u;
    // the segment is elements [lo, hi) of the group's own numbering
    const int32_t lo = (int32_t)r - 4 * (int32_t)u, hi = (int32_t)(cg.inner + r) - 4 * (int32_t)u;
    const uint32_t below_hi = hi >= 4 ? 0xFu : hi <= 0 ? 0u : (1u << hi) - 1u;
    const uint32_t from_lo = lo <= 0 ? 0xFu : (0xFu << lo) & 0xFu;
    mask = below_hi & from_lo;
}

__device__ __forceinline__ uint32_t ragged_slice_slots(const RaggedClusterGeom& cg, uint32_t s)
{
    const uint32_t t0 = s * cg.slice_groups;
    if (t0 >= cg.block_groups) return 0u;
    return cg.block_groups - t0 < cg.slice_groups ? cg.block_groups - t0 : cg.slice_groups;
}

__device__ __forceinline__ uint4 keep_masked(const uint4& v, uint32_t mask)
{
    return make_uint4((mask & 1u) ? v.x : 0u, (mask & 2u) ? v.y : 0u, (mask & 4u) ? v.z : 0u, (mask & 8u) ? v.w : 0u);
}

template <int MODE>
__global__ __launch_bounds__(kThreads, 4) void block_cluster_ragged_kernel(const uint32_t* in, uint32_t* out, uint32_t* slots,
                                                                           RaggedClusterGeom cg, int wl, int symmetric,
                                                                           RngKey key)
{
    constexpr int GPT = 16;
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? 9 : 0;          // random words parked in LDS, as in the kernels above
    __shared__ uint4 parked[PRE > 0 ? PRE * kThreads : 1];
    __shared__ uint32_t lds[kThreads / 64];
    __shared__ uint32_t shared_word;
    const uint32_t wg = (uint32_t)linear_block();
    if (wg >= cg.total_wgs) return;                                // the whole workgroup leaves together
    const uint32_t b = wg / cg.slices, s = wg - b * cg.slices;
    const uint32_t t0 = s * cg.slice_groups;
    const uint32_t nslots = ragged_slice_slots(cg, s);
    const bool short_tail = (cg.n & 3u) != 0u;                     // the array's last group is not whole

    // Every load is one unconditional dwordx4 inside the array, so that all sixteen are in flight
    // together: an unused slot reads the group before it, and the array's short last group reads
    // the array's last four elements instead (put right below, `shift` elements further on).
    uint4 v[GPT];
    uint32_t shifts = 0u;
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        if (t < nslots) {
            uint64_t j;
            uint32_t mask;
            ragged_slot(cg, b, t0 + t, j, mask);
            uint64_t at = 4u * j;
            if (mask == 0u) at -= 4u;
            if (at + 4u > cg.n) {
                shifts |= (uint32_t)(at + 4u - cg.n) << (2 * k);
                at = cg.n - 4u;
            }
            v[k] = to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4_at_dword*>(in + at)));
            if (k < PRE) {
                const Words4 r = random_words(j, key, 0u);
                parked[k * kThreads + threadIdx.x] = make_uint4(r.w[0], r.w[1], r.w[2], r.w[3]);
            }
        }
    }
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        // (the slot is worked out again, here and below, rather than kept: sixteen group numbers and
        // masks do not fit the registers next to sixteen groups; the empty asm keeps the compiler from
        // finding out that it is the same computation)
        uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        asm volatile("" : "+v"(t));
        uint32_t mask = 0u;
        if (t < nslots) {
            uint64_t j;
            ragged_slot(cg, b, t0 + t, j, mask);
        }
        if (short_tail) {
            const uint32_t sh = (shifts >> (2 * k)) & 3u;          // element e of the group was loaded as word e + sh
            if (sh == 1u) v[k] = make_uint4(v[k].y, v[k].z, v[k].w, 0u);
            else if (sh == 2u) v[k] = make_uint4(v[k].z, v[k].w, 0u, 0u);
            else if (sh == 3u) v[k] = make_uint4(v[k].w, 0u, 0u, 0u);
        }
        const uint32_t gm = max4_mag(keep_masked(v[k], mask));       // strangers stay in v[k]: quantized below, never stored
        m = m > gm ? m : gm;
    }
    m = workgroup_max(m, lds);

    uint32_t* mine = slots + (uint64_t)b * cg.slices;
    const uint32_t bm = meet_in_block(mine, s, cg.slices, m, cg.wait_us, lds, shared_word, [&](uint32_t i) {
        // slice i of this block from memory, element by element where a group is shared
        uint32_t own = 0;
        const uint32_t count = ragged_slice_slots(cg, i);
        for (uint32_t t = threadIdx.x; t < count; t += kThreads) {
            uint64_t j;
            uint32_t mask;
            ragged_slot(cg, b, i * cg.slice_groups + t, j, mask);
#pragma unroll
            for (uint32_t e = 0; e < 4u; ++e) {
                if (mask & (1u << e)) {
                    const uint32_t a = in[4u * j + e] & 0x7fffffffu;
                    own = own > a ? own : a;
                }
            }
        }
        return own;
    });

    const GridPlan p = block_plan(bm, wl, symmetric);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        asm volatile("" : "+v"(t));
        if (t < nslots) {
            uint64_t j;
            uint32_t mask;
            ragged_slot(cg, b, t0 + t, j, mask);
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) {
                const uint4 w = parked[k * kThreads + threadIdx.x];
                r = Words4{{w.x, w.y, w.z, w.w}};
            } else if (MODE == QSIM_STOCHASTIC) {
                r = random_words(j, key, 0u);
            }
            const uint4 q = quantize_group_to_grid<MODE>(v[k], p, r);
            uint32_t* dst = out + 4u * j;
            if (mask == 0xFu) {
                __builtin_nontemporal_store(to_u32x4(q), reinterpret_cast<u32x4_at_dword*>(dst));
            } else {
                if (mask & 1u) dst[0] = q.x;
                if (mask & 2u) dst[1] = q.y;
                if (mask & 4u) dst[2] = q.z;
                if (mask & 8u) dst[3] = q.w;
            }
        }
    }
}

// Blocks along an inner dimension that are SHORT (outer * inner <= 2048 elements, inner % 4 == 0,
// aligned arrays): a [2, 300000, 64] tensor with one block per index of the middle dimension.  One
// workgroup takes as many consecutive blocks as fit 4096 elements and holds them in registers, four
// groups per thread; block maxima meet in LDS; single pass, nothing to wait for.  For a fixed outer
// index the segments of consecutive blocks are neighbours in memory, so the accesses of a workgroup
// fall into `outer` contiguous runs.
struct StridedPackedGeom {
    uint64_t nblocks;
    uint32_t outer_inner;      // elements per block, a multiple of 4, at most 2048
    uint32_t groups_per_block; // outer_inner / 4
    uint32_t magic_groups;     // floor(2^32 / groups_per_block) + 1 (unused when groups_per_block == 1)
    uint32_t inner;
    uint32_t magic_inner;      // floor(2^32 / inner) + 1
    uint32_t blocks_per_wg;    // floor(1024 / groups_per_block), at least 2
};

template <int MODE>
__global__ __launch_bounds__(kThreads) void block_strided_packed_kernel(const uint32_t* in, uint32_t* out, StridedPackedGeom pg,
                                                                        int wl, int symmetric, RngKey key)
{
    constexpr int GPT = 4;
    __shared__ uint32_t blockmax[kThreads * GPT];                 // at most 1024 blocks of one group each
    const uint64_t b0 = linear_block() * pg.blocks_per_wg;
    if (b0 >= pg.nblocks) return;                                 // the whole workgroup leaves together
    const uint32_t mine = pg.nblocks - b0 < pg.blocks_per_wg ? (uint32_t)(pg.nblocks - b0) : pg.blocks_per_wg;
    const uint32_t ngroups = mine * pg.groups_per_block;          // at most 1024
    for (uint32_t t = threadIdx.x; t < mine; t += kThreads) blockmax[t] = 0u;
    __syncthreads();

    uint4 v[GPT];
    uint32_t owner[GPT];
    uint64_t where[GPT];
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        owner[k] = 0u;
        where[k] = 0u;
        if (t < ngroups) {
            const uint32_t bl = pg.groups_per_block == 1u ? t : __umulhi(t, pg.magic_groups);     // exact: t < 2^16
            const uint32_t tt = (t - bl * pg.groups_per_block) * 4u;                              // element within the block
            const uint32_t o = __umulhi(tt, pg.magic_inner);                                       // exact: tt < 2^16
            const uint32_t i = tt - o * pg.inner;
            owner[k] = bl;
            where[k] = (((uint64_t)o * pg.nblocks + (b0 + bl)) * pg.inner + i) >> 2;
            v[k] = to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(in) + where[k]));
        }
    }
    // stochastic rounding: the random words are drawn while the loads are in flight
    Words4 words[MODE == QSIM_STOCHASTIC ? GPT : 1];
    if (MODE == QSIM_STOCHASTIC) {
#pragma unroll
        for (int k = 0; k < GPT; ++k) {
            words[k] = random_words(where[k], key, 0u);
            asm volatile("" : "+v"(words[k].w[0]), "+v"(words[k].w[1]), "+v"(words[k].w[2]), "+v"(words[k].w[3]));
        }
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        if (t < ngroups) atomicMax(&blockmax[owner[k]], max4_mag(v[k]));
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        if (t < ngroups) {
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (MODE == QSIM_STOCHASTIC) r = words[k];
            const GridPlan p = block_plan(blockmax[owner[k]], wl, symmetric);
            __builtin_nontemporal_store(to_u32x4(quantize_group_to_grid<MODE>(v[k], p, r)), reinterpret_cast<u32x4*>(out) + where[k]);
        }
    }
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
