// Block floating point, contiguous blocks that fit the registers of one team or workgroup:
// read once, reduce, quantize, write once.
#pragma once

#include "qsim_kernel_common.hpp"

namespace qsim {

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
    const bool finite = wave_plans_are_finite<MODE>(p);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = lane + (uint32_t)k * stride;
        if (t < groups) {
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) r = early[k];
            else if (MODE == QSIM_STOCHASTIC) r = random_words(j0 + (g0 + t), key, 0u);
            store_group<true>(wout, (uint64_t)(g0 + t), (uint64_t)end, quantize_group_of_block<MODE>(v[k], p, r, finite));
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
    int all_finite = 1;
    for (uint32_t t = threadIdx.x; t < nrows; t += kThreads)
        if (!plan_is_finite<MODE>(block_plan(rowmax[t], wl, symmetric))) all_finite = 0;
    // none of the workgroup's blocks holds Inf or NaN (nearly always): the table then holds exponent
    // fields, from which a plan per element is cheap
    const bool finite = __syncthreads_and(all_finite) != 0;
    if (finite) {
        for (uint32_t t = threadIdx.x; t < nrows; t += kThreads) rowmax[t] = clamped_field23(rowmax[t]);
        __syncthreads();
    }
    const FieldPlan fp = field_plan(wl, symmetric);
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
            for (int e = 0; e < 4; ++e) {
                const uint32_t entry = rowmax[row[e]];
                o[e] = finite ? quantize_finite_to_grid<MODE>(bits[e], plan_of_field(entry, fp), r.w[e])
                              : quantize_to_grid<MODE>(bits[e], block_plan(entry, wl, symmetric), r.w[e]);
            }
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

// The same for SHORT blocks along an inner dimension whose segments are not whole groups, or in arrays
// that are only dword aligned ([2, 100000, 154] with one block per middle index; per-channel blocks
// of a small batch of 7 x 7 maps): a workgroup owns `rows_per_wg` consecutive blocks, whose segments
// are neighbours in memory for a fixed outer index: `outer` contiguous runs, each walked in the
// array's own groups like the single range of block_ragged_kernel.  Every run is given `run_slots`
// group slots, the most it can cover at any alignment; slot t of the workgroup is slot t mod
// run_slots of run t div run_slots (unused when the run covers fewer groups).  One pass, one launch.
struct RaggedRunsGeom {
    uint64_t n, nblocks;
    uint32_t outer, inner;
    uint32_t rows_per_wg;      // at most kRaggedMaxRows; rows_per_wg * inner < 2^16
    uint32_t run_slots;        // (rows_per_wg * inner + 6) / 4 + 1 ... outer * run_slots <= kThreads * GPT
    uint32_t magic_slots;      // floor(2^32 / run_slots) + 1
    uint32_t magic_inner;      // floor(2^32 / inner) + 1 (any value when inner == 1)
};

template <int MODE, int GPT>
__global__ __launch_bounds__(kThreads) void block_ragged_runs_kernel(const uint32_t* in, uint32_t* out, RaggedRunsGeom rg, int wl,
                                                                     int symmetric, RngKey key)
{
    __shared__ uint32_t rowmax[kRaggedMaxRows];
    const uint64_t r0 = linear_block() * rg.rows_per_wg;
    if (r0 >= rg.nblocks) return;                     // the whole workgroup leaves together
    const uint32_t nrows = rg.nblocks - r0 < rg.rows_per_wg ? (uint32_t)(rg.nblocks - r0) : rg.rows_per_wg;
    const uint32_t span = nrows * rg.inner;           // elements of one run
    const uint32_t nslots = rg.outer * rg.run_slots;
    const uint32_t inner = rg.inner;

    for (uint32_t t = threadIdx.x; t < nrows; t += kThreads) rowmax[t] = 0u;
    __syncthreads();

    // slot t: its group in the array, and how many elements of the run's first group come before the run
    auto slot = [&](uint32_t t, uint64_t& j, uint32_t& u, uint32_t& lead) {
        const uint32_t o = __umulhi(t, rg.magic_slots);                  // exact: t < 2^16
        u = t - o * rg.run_slots;
        const uint64_t e0 = ((uint64_t)o * rg.nblocks + r0) * inner;    // first element of the run
        lead = (uint32_t)e0 & 3u;
        j = (e0 >> 2) + u;
    };

    uint4 v[GPT];
    uint32_t rows01[GPT], rows23[GPT];       // block of each element relative to r0, 16 bits each (clamped outside the run)
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? (GPT < 4 ? GPT : 4) : 0;
    Words4 early[PRE > 0 ? PRE : 1];         // random words of the first groups, drawn while the loads are in flight
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        if (t < nslots) {
            uint64_t j;
            uint32_t u, lead;
            slot(t, j, u, lead);
            if (4u * u < lead + span) v[k] = load_group<false>(in, j, rg.n);
            if (k < PRE) {
                early[k < PRE ? k : 0] = random_words(j, key, 0u);
                asm volatile("" : "+v"(early[k < PRE ? k : 0].w[0]), "+v"(early[k < PRE ? k : 0].w[1]),
                             "+v"(early[k < PRE ? k : 0].w[2]), "+v"(early[k < PRE ? k : 0].w[3]));
            }
        }
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        rows01[k] = rows23[k] = 0u;
        if (t < nslots) {
            uint64_t j;
            uint32_t u, lead;
            slot(t, j, u, lead);
            const uint32_t bits[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
            uint32_t mag[4], row[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t at = u * 4u + (uint32_t)e;                  // offset from the start of the run's first group
                const bool mine = at >= lead && at - lead < span;
                const uint32_t off = mine ? at - lead : 0u;
                const uint32_t r = inner == 1u ? off : __umulhi(off, rg.magic_inner);
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
    int all_finite = 1;
    for (uint32_t t = threadIdx.x; t < nrows; t += kThreads)
        if (!plan_is_finite<MODE>(block_plan(rowmax[t], wl, symmetric))) all_finite = 0;
    const bool finite = __syncthreads_and(all_finite) != 0;      // as in block_ragged_kernel
    if (finite) {
        for (uint32_t t = threadIdx.x; t < nrows; t += kThreads) rowmax[t] = clamped_field23(rowmax[t]);
        __syncthreads();
    }
    const FieldPlan fp = field_plan(wl, symmetric);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        if (t < nslots) {
            uint64_t j;
            uint32_t u, lead;
            slot(t, j, u, lead);
            const uint32_t at = u * 4u;
            if (at < lead + span) {                                       // (a slot past the run's last group holds nothing)
                Words4 r = {{0u, 0u, 0u, 0u}};
                if (k < PRE) r = early[k < PRE ? k : 0];
                else if (MODE == QSIM_STOCHASTIC) r = random_words(j, key, 0u);
                const uint32_t bits[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
                const uint32_t row[4] = {rows01[k] & 0xffffu, rows01[k] >> 16, rows23[k] & 0xffffu, rows23[k] >> 16};
                uint32_t o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t entry = rowmax[row[e]];
                    o[e] = finite ? quantize_finite_to_grid<MODE>(bits[e], plan_of_field(entry, fp), r.w[e])
                                  : quantize_to_grid<MODE>(bits[e], block_plan(entry, wl, symmetric), r.w[e]);
                }
                if (at >= lead && at + 3u - lead < span) {
                    store_group<false>(out, j, rg.n, make_uint4(o[0], o[1], o[2], o[3]));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (at + (uint32_t)e >= lead && at + (uint32_t)e - lead < span) out[j * 4 + (uint64_t)e] = o[e];
                }
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
    const bool finite = wave_plans_are_finite<MODE>(p);
    for (uint64_t t = threadIdx.x; t < len; t += kThreads) {
        const uint64_t i = start + t;
        uint32_t r = 0;
        if (MODE == QSIM_STOCHASTIC) r = random_words(i >> 2, key, 0u).w[i & 3];
        out[i] = finite ? quantize_finite_to_grid<MODE>(in[i], p, r) : quantize_to_grid<MODE>(in[i], p, r);
    }
}

}  // namespace qsim
