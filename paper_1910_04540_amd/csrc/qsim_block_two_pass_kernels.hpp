// Block floating point in two passes over memory (maxima, then quantize): the general form for any
// layout, the column and flat forms for blocks along an inner dimension, the streaming form for
// long contiguous blocks.
#pragma once

#include "qsim_kernel_common.hpp"

namespace qsim {

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
    const bool finite = wave_plans_are_finite<MODE>(p);
    const uint64_t len = block_length(sg, b);
    const uint64_t t0 = (uint64_t)blockIdx.y * sg.slice_len;
    const uint64_t t1 = (t0 + sg.slice_len < len) ? t0 + sg.slice_len : len;
    if (VEC) {
        for (uint64_t t = t0 + 4ull * threadIdx.x; t < t1; t += 4ull * kThreads) {
            const uint64_t j = flat_index(sg.g, b, t) / 4;
            const uint4 v = load_group<true>(in, j, sg.g.n);
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (MODE == QSIM_STOCHASTIC) r = random_words(j, key, 0u);
            store_group<true>(out, j, sg.g.n, quantize_group_of_block<MODE>(v, p, r, finite));
        }
    } else {
        for (uint64_t t = t0 + 4ull * threadIdx.x; t < t1; t += 4ull * kThreads) {
            const uint64_t o = sg.g.outer == 1 ? 0 : segment_of(sg.g, t), i = t - o * sg.g.inner;
            if (t + 4 <= t1 && (sg.g.outer == 1 || i + 4 <= sg.g.inner)) {
                const uint64_t at = sg.g.outer == 1 ? b * sg.g.inner + t : (o * sg.g.nblocks + b) * sg.g.inner + i;
                const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_at_dword*>(in + at));
                Words4 r = {{0u, 0u, 0u, 0u}};
                if (MODE == QSIM_STOCHASTIC) r = random_words_at(at, key, 0u);
                __builtin_nontemporal_store(to_u32x4(quantize_group_of_block<MODE>(to_uint4(w), p, r, finite)),
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
    uint32_t stream_first;     // pass 1 reads with non-temporal loads: the tensor is too large for pass 2 to find it cached
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
                        if (o + k < o1) v[k] = column_load<ALIGNED>(in, (o + k) * cg.row + 4ull * c, have, cg.stream_first != 0u);
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

// `parts` > 0 (blocks of one column only): the block maxima are not folded yet; colparts holds
// `parts` rows of column maxima and the thread folds the entries of its own four columns, which
// saves the launch of a fold kernel.
constexpr uint32_t kColumnSharedRuns = 63;     // runs per wavefront when neighbouring lanes share Philox blocks

template <int MODE, bool ALIGNED>
__global__ __launch_bounds__(kThreads) void block_column_apply_kernel(const uint32_t* in, uint32_t* out,
                                                                      const uint32_t* blockmax, const uint4* colparts,
                                                                      uint32_t parts, ColumnGeom cg, int wl, int symmetric,
                                                                      RngKey key)
{
    // Stochastic rounding of runs that are not group-aligned needs two Philox blocks per run, the
    // second of which is the next run's first: there a wavefront takes 63 runs, its last lane draws
    // the 64th block only, and every lane gets its second block from its neighbour (SHARE).
    constexpr bool SHARE = MODE == QSIM_STOCHASTIC && !ALIGNED;
    uint32_t c = blockIdx.x * kThreads + threadIdx.x;
    bool live = true;
    if (SHARE) {
        const uint32_t lane = threadIdx.x & 63u;
        c = (blockIdx.x * (kThreads / 64u) + (threadIdx.x >> 6)) * kColumnSharedRuns + lane;
        if (c - lane >= cg.row_groups) return;                       // the whole wavefront leaves together
        live = lane < kColumnSharedRuns && c < cg.row_groups;
    } else if (c >= cg.row_groups) {
        return;
    }
    const uint64_t o0 = (uint64_t)blockIdx.y * cg.rows_per_slice;
    const uint64_t o1 = (o0 + cg.rows_per_slice < cg.outer) ? o0 + cg.rows_per_slice : cg.outer;
    const uint32_t have = live ? cg.row - 4u * c : 0u;               // 0: no loads, no stores
    const uint32_t cp = c < cg.row_groups ? c : cg.row_groups - 1u;  // (a lane without elements reads a valid plan)
    GridPlan p[4];
    if (parts > 0u) {
        uint4 m = colparts[cp];
        for (uint32_t s = 1; s < parts; ++s) {
            const uint4 a = colparts[(uint64_t)s * cg.row_groups + cp];
            m.x = m.x > a.x ? m.x : a.x;
            m.y = m.y > a.y ? m.y : a.y;
            m.z = m.z > a.z ? m.z : a.z;
            m.w = m.w > a.w ? m.w : a.w;
        }
        p[0] = block_plan(m.x, wl, symmetric);
        p[1] = block_plan(m.y, wl, symmetric);
        p[2] = block_plan(m.z, wl, symmetric);
        p[3] = block_plan(m.w, wl, symmetric);
    } else if (cg.inner % 4 == 0) {
        p[0] = p[1] = p[2] = p[3] = block_plan(blockmax[(4u * cp) / cg.inner], wl, symmetric);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t col = 4u * cp + (uint32_t)e < cg.row ? 4u * cp + (uint32_t)e : cg.row - 1u;
            p[e] = block_plan(blockmax[col / cg.inner], wl, symmetric);
        }
    }
    const bool finite = __all(plan_is_finite<MODE>(p[0]) && plan_is_finite<MODE>(p[1]) && plan_is_finite<MODE>(p[2]) &&
                              plan_is_finite<MODE>(p[3]) ? 1 : 0) != 0;
    // (four rows at a time; keeping the loads of the next four in flight meanwhile, as the flat form
    // does, measured 3-5 % slower here)
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
                if (MODE == QSIM_STOCHASTIC) r = ALIGNED ? random_words(at >> 2, key, 0u) : random_words_at_shared(at, key, 0u);
                uint4 q;
                if (finite) {
                    q.x = quantize_finite_to_grid<MODE>(v[k].x, p[0], r.w[0]);
                    q.y = quantize_finite_to_grid<MODE>(v[k].y, p[1], r.w[1]);
                    q.z = quantize_finite_to_grid<MODE>(v[k].z, p[2], r.w[2]);
                    q.w = quantize_finite_to_grid<MODE>(v[k].w, p[3], r.w[3]);
                } else {
                    q.x = quantize_to_grid<MODE>(v[k].x, p[0], r.w[0]);
                    q.y = quantize_to_grid<MODE>(v[k].y, p[1], r.w[1]);
                    q.z = quantize_to_grid<MODE>(v[k].z, p[2], r.w[2]);
                    q.w = quantize_to_grid<MODE>(v[k].w, p[3], r.w[3]);
                }
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
// collected in an LDS table per workgroup (ds_max), written out as partial[workgroup][block],
// folded by one launch of block_fold_rows_once_kernel, and pass 2 walks the same ranges with the
// finished maxima in LDS.
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
    uint32_t copies;             // copies of the LDS table in pass 1: a power of two, 1..64; copies * (nblocks rounded up to 4) <= 4096
    uint32_t stream_first;       // pass 1 reads with non-temporal loads (see ColumnGeom)
};

// Where block t sits in a table in LDS.  A lane's four elements are neighbours, so with inner == 1
// the lanes of a wavefront ask for entries 4 * lane + e in one instruction: eight LDS banks out of
// 32.  Moving the entry within its aligned run of four, by bits 5 and 6 of its number, spreads a
// half-wavefront over all banks.
__device__ __forceinline__ uint32_t flat_slot(uint32_t t) { return t ^ ((t >> 5) & 3u); }

__device__ __forceinline__ uint32_t flat_block(const FlatGeom& fg, uint32_t pos /* < 2^16 */)
{
    const uint32_t in_row = fg.row == 1u ? 0u : pos - __umulhi(pos, fg.magic_row) * fg.row;
    return fg.inner == 1u ? in_row : __umulhi(in_row, fg.magic_inner);
}

// The blocks of the four elements from position pos on: one reduction modulo the row, then steps of one.
__device__ __forceinline__ void flat_blocks4(const FlatGeom& fg, uint32_t pos /* < 2^16 - 3 */, uint32_t (&b)[4])
{
    if (fg.row < 4u) {                                   // (uniform) four elements may wrap around more than once
#pragma unroll
        for (uint32_t e = 0; e < 4u; ++e) b[e] = flat_block(fg, pos + e);
        return;
    }
    const uint32_t r0 = pos - __umulhi(pos, fg.magic_row) * fg.row;
#pragma unroll
    for (uint32_t e = 0; e < 4u; ++e) {
        uint32_t r = r0 + e;
        r = r >= fg.row ? r - fg.row : r;
        b[e] = fg.inner == 1u ? r : __umulhi(r, fg.magic_inner);
    }
}

// The groups of one step.  A step that lies wholly inside the array (all but the last) issues its
// loads back to back with nothing in between, so that all of them are in flight together.
template <bool STREAM>
__device__ __forceinline__ void flat_load_step(const uint32_t* in, uint64_t base, const FlatGeom& fg, uint4 (&v)[kFlatGpt])
{
    if ((base + kFlatStepGroups) * 4 <= fg.n) {                              // wave-uniform
        const u32x4_at_dword* p = reinterpret_cast<const u32x4_at_dword*>(in + base * 4) + threadIdx.x;
#pragma unroll
        for (int k = 0; k < kFlatGpt; ++k) {
            const u32x4 w = STREAM ? __builtin_nontemporal_load(p + k * kThreads) : p[k * kThreads];
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

__global__ __launch_bounds__(kThreads) void block_flat_max_kernel(const uint32_t* in, uint32_t* partial, uint32_t* blockmax,
                                                                  FlatGeom fg)
{
    // (the fold that follows brings its results in with atomic maxima: the table they meet in starts at zero)
    if (blockIdx.x == 0)
        for (uint32_t t = threadIdx.x; t < fg.nblocks; t += kThreads) blockmax[t] = 0u;
    // Few blocks mean many lanes per block, and same-address LDS atomics of one instruction are
    // carried out one after the other: so the table is replicated, lane l works on copy l mod copies
    // (copies * nblocks, rounded up to four, <= 4096), and the copies are folded at the end.
    __shared__ uint32_t table[kFlatMaxBlocks];
    const uint32_t copies = fg.copies;
    const uint32_t room = (fg.nblocks + 3u) & ~3u;                  // of one copy: flat_slot stays within runs of four
    for (uint32_t t = threadIdx.x; t < room * copies; t += kThreads) table[t] = 0u;
    __syncthreads();
    uint32_t* mine = table + (threadIdx.x & (copies - 1u)) * room;
    // steps are dealt out round-robin, so that at any moment the workgroups together read one
    // contiguous front of the tensor; the loads of a workgroup's next step are under way while it
    // works on this one
    const uint64_t g1 = fg.groups, stride = (uint64_t)fg.wgs * kFlatStepGroups;
    auto load = [&](uint64_t base, uint4 (&v)[kFlatGpt]) {
        if (fg.stream_first) flat_load_step<true>(in, base, fg, v);                   // wave-uniform
        else flat_load_step<false>(in, base, fg, v);
    };
    auto fold = [&](uint64_t base, const uint4 (&v)[kFlatGpt]) {
        const uint32_t pos0 = (uint32_t)((base * 4) % fg.row);            // wave-uniform
#pragma unroll
        for (int k = 0; k < kFlatGpt; ++k) {
            const uint64_t j = base + threadIdx.x + (uint64_t)k * kThreads;
            if (j < g1) {
                const uint32_t off = (threadIdx.x + (uint32_t)k * kThreads) * 4u;
                if (fg.inner % 4u == 0u) {                                    // a group never straddles blocks
                    atomicMax(&mine[flat_slot(flat_block(fg, pos0 + off))], max4_mag(v[k]));
                } else {
                    const uint32_t mag[4] = {v[k].x & 0x7fffffffu, v[k].y & 0x7fffffffu, v[k].z & 0x7fffffffu,
                                             v[k].w & 0x7fffffffu};
                    uint32_t b[4];                                            // (elements past the end read as zero; their block number is still a valid one)
                    flat_blocks4(fg, pos0 + off, b);
                    uint32_t prev = b[0], m = mag[0];
#pragma unroll
                    for (uint32_t e = 1; e < 4; ++e) {
                        if (b[e] != prev) {
                            atomicMax(&mine[flat_slot(prev)], m);
                            m = 0u;
                            prev = b[e];
                        }
                        m = m > mag[e] ? m : mag[e];
                    }
                    atomicMax(&mine[flat_slot(prev)], m);
                }
            }
        }
    };
    // (two sets of registers take turns, so that nothing waits for the loads of the step ahead)
    uint64_t base = (uint64_t)blockIdx.x * kFlatStepGroups;
    uint4 even[kFlatGpt], odd[kFlatGpt];
    if (base < g1) load(base, even);
    while (base < g1) {
        const uint64_t second = base + stride, third = second + stride;
        if (second < g1) load(second, odd);
        fold(base, even);
        if (second >= g1) break;
        if (third < g1) load(third, even);
        fold(second, odd);
        base = third;
    }
    __syncthreads();
    for (uint32_t t = threadIdx.x; t < fg.nblocks; t += kThreads) {
        uint32_t m = table[flat_slot(t)];
        for (uint32_t c = 1; c < copies; ++c) {
            const uint32_t a = table[c * room + flat_slot(t)];
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

// blockmax[b] = max over all `rows` rows k of src[k * nblocks + b] in ONE launch, for any number of
// rows: workgroup (x, y) takes 32 neighbouring blocks (one cache line of a row) and 64 rows, eight
// rows per thread, all eight loads in flight; the eight parts meet in LDS and the result joins
// blockmax[b] by one atomic maximum (rows / 64 of them per block).  blockmax must hold zeros.
constexpr uint32_t kFoldOnceRows = 64;

__global__ __launch_bounds__(kThreads) void block_fold_rows_once_kernel(const uint32_t* src, uint32_t* blockmax, uint32_t nblocks,
                                                                        uint32_t rows)
{
    __shared__ uint32_t part[kThreads / 32][32];
    const uint32_t c = threadIdx.x & 31u, p = threadIdx.x >> 5;
    const uint32_t b = blockIdx.x * 32u + c;
    const uint32_t k0 = blockIdx.y * kFoldOnceRows + p * 8u;
    uint32_t a[8];
#pragma unroll
    for (uint32_t k = 0; k < 8u; ++k) a[k] = b < nblocks && k0 + k < rows ? src[(uint64_t)(k0 + k) * nblocks + b] : 0u;
    uint32_t m = 0;
#pragma unroll
    for (uint32_t k = 0; k < 8u; ++k) m = m > a[k] ? m : a[k];
    part[p][c] = m;
    __syncthreads();
    if (p == 0u && b < nblocks) {
#pragma unroll
        for (uint32_t q = 1; q < kThreads / 32; ++q) m = m > part[q][c] ? m : part[q][c];
        if (m != 0u) __hip_atomic_fetch_max(&blockmax[b], m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int MODE>
__global__ __launch_bounds__(kThreads) void block_flat_apply_kernel(const uint32_t* in, uint32_t* out, const uint32_t* blockmax,
                                                                    FlatGeom fg, int wl, int symmetric, RngKey key)
{
    __shared__ uint32_t table[kFlatMaxBlocks];
    int all_finite = 1;
    for (uint32_t t = threadIdx.x; t < fg.nblocks; t += kThreads) {
        const uint32_t m = blockmax[t];
        table[flat_slot(t)] = m;
        if (!plan_is_finite<MODE>(block_plan(m, wl, symmetric))) all_finite = 0;
    }
    // no block of the tensor holds Inf or NaN (nearly always): the table then holds exponent fields,
    // from which a plan per element is cheap
    const bool finite = __syncthreads_and(all_finite) != 0;
    if (finite) {
        for (uint32_t t = threadIdx.x; t < fg.nblocks; t += kThreads) table[flat_slot(t)] = clamped_field23(table[flat_slot(t)]);
        __syncthreads();
    }
    const FieldPlan fp = field_plan(wl, symmetric);
    // steps are dealt out round-robin, so that at any moment the workgroups together read one
    // contiguous front of the tensor; the loads of a workgroup's next step are under way while it
    // works on this one
    const uint64_t g1 = fg.groups, stride = (uint64_t)fg.wgs * kFlatStepGroups;
    auto apply = [&](uint64_t base, const uint4 (&v)[kFlatGpt]) {
        const uint32_t pos0 = (uint32_t)((base * 4) % fg.row);            // wave-uniform
#pragma unroll
        for (int k = 0; k < kFlatGpt; ++k) {
            const uint64_t j = base + threadIdx.x + (uint64_t)k * kThreads;
            if (j < g1) {
                const uint32_t off = (threadIdx.x + (uint32_t)k * kThreads) * 4u;
                Words4 r = {{0u, 0u, 0u, 0u}};
                if (MODE == QSIM_STOCHASTIC) r = random_words(j, key, 0u);
                uint4 o;
                if (fg.inner % 4u == 0u) {
                    const uint32_t entry = table[flat_slot(flat_block(fg, pos0 + off))];
                    o = finite ? quantize_group_of_block<MODE>(v[k], plan_of_field(entry, fp), r, true)
                               : quantize_group_to_grid<MODE>(v[k], block_plan(entry, wl, symmetric), r);
                } else {
                    uint32_t b[4];
                    flat_blocks4(fg, pos0 + off, b);
                    if (finite) {
                        o.x = quantize_finite_to_grid<MODE>(v[k].x, plan_of_field(table[flat_slot(b[0])], fp), r.w[0]);
                        o.y = quantize_finite_to_grid<MODE>(v[k].y, plan_of_field(table[flat_slot(b[1])], fp), r.w[1]);
                        o.z = quantize_finite_to_grid<MODE>(v[k].z, plan_of_field(table[flat_slot(b[2])], fp), r.w[2]);
                        o.w = quantize_finite_to_grid<MODE>(v[k].w, plan_of_field(table[flat_slot(b[3])], fp), r.w[3]);
                    } else {
                        o.x = quantize_to_grid<MODE>(v[k].x, block_plan(table[flat_slot(b[0])], wl, symmetric), r.w[0]);
                        o.y = quantize_to_grid<MODE>(v[k].y, block_plan(table[flat_slot(b[1])], wl, symmetric), r.w[1]);
                        o.z = quantize_to_grid<MODE>(v[k].z, block_plan(table[flat_slot(b[2])], wl, symmetric), r.w[2]);
                        o.w = quantize_to_grid<MODE>(v[k].w, block_plan(table[flat_slot(b[3])], wl, symmetric), r.w[3]);
                    }
                }
                store_group<false>(out, j, fg.n, o);
            }
        }
    };
    // (two sets of registers take turns, so that nothing waits for the loads of the step ahead)
    uint64_t base = (uint64_t)blockIdx.x * kFlatStepGroups;
    uint4 even[kFlatGpt], odd[kFlatGpt];
    if (base < g1) flat_load_step<true>(in, base, fg, even);
    while (base < g1) {
        const uint64_t second = base + stride, third = second + stride;
        if (second < g1) flat_load_step<true>(in, second, fg, odd);
        apply(base, even);
        if (second >= g1) break;
        if (third < g1) flat_load_step<true>(in, third, fg, even);
        apply(second, odd);
        base = third;
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

// The same with one load in flight and few registers: for the rarely taken paths of kernels that
// hold a slice of their own in registers meanwhile.
__device__ __forceinline__ uint32_t slice_max_frugal(const uint32_t* in, const SliceView& sv)
{
    uint32_t m = 0;
    for (uint64_t t = threadIdx.x; t < sv.groups; t += blockDim.x) {       // (workgroups of 256 or 512 threads)
        const uint32_t gm = max4_mag(load_group<false>(in, sv.j0 + t, sv.end));
        m = m > gm ? m : gm;
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
        const bool finite = wave_plans_are_finite<MODE>(p);
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
                    store_group<true>(out, sv.j0 + t, sv.end, quantize_group_of_block<MODE>(v[k], p, r, finite));
                }
            }
        }
    }
}

}  // namespace qsim
