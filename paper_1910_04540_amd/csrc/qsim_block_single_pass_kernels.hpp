// Block floating point in a single pass for blocks larger than one workgroup: the workgroups hold
// the data in registers and meet over their maxima (whole tensor, block by block for contiguous rows
// and for blocks along an inner dimension), and several short strided blocks per workgroup.
#pragma once

#include "qsim_kernel_common.hpp"
#include "qsim_block_two_pass_kernels.hpp"

namespace qsim {

// ---------------------------------------------------------------------------------------------
// The meeting.  The workgroups that hold the slices of one block each know the largest magnitude of
// their slice and need the largest of the block.  They count themselves into counters that carry the
// running maximum along; the last to arrive publishes the block's maximum in flags the others poll.
//
// Scratch: 64-bit words of device memory.  All communication is through relaxed device-scope
// atomics on words only atomics touch: nothing else has to become visible between workgroups, so no
// release or acquire fence (each of which writes back or invalidates a whole L2 on this multi-die
// part) is needed; order is kept by waiting for the returned value of one atomic before the next one
// is issued.  The words (`stride` apart, 16 = a 128-byte line each while they are few, so that no
// address sees more than a few dozen operations: a single word polled by a thousand workgroups
// serialises at its memory channel and costs more than the kernel's whole memory traffic):
//   word 0                                      workgroups that gave up waiting (statistics only)
//   word 1                                      the epoch: number of the last launch that met here
//   word 2                                      groups of 256 blocks whose meetings are over
//   counters (must be zero when a launch starts, and are zero again when it ends)
//     counter of group q = b * groups + s / 32  low half: largest magnitude so far; high half: arrivals.
//                                               A workgroup first folds its maximum in, waits for that
//                                               to be done, then counts itself; so the one that counts
//                                               last reads the group's final maximum with its count,
//                                               and puts the counter back to zero.
//     top counter of block b                    the same over the groups of a block (groups > 1)
//     (forms that poll slots instead, see meet_in_block: one counter per block, arrivals only)
//     blocks whose meetings are over            one word per 256 blocks
//   tagged words (count only when their high half is this launch's tag = epoch + 1; never cleaned)
//     flag of group q                           tag << 32 | published | the block's maximum: written by
//                                               the last arrival of the block, polled by the group
//     slot of workgroup w                       tag << 32 | published | its maximum: read only by a
//                                               workgroup whose wait ran out
// Every workgroup reads the epoch before anything else; the last arrival of the last block, which
// knows that everybody has read it, stores the new one.  So a scratch that is all zero before its
// first launch stays usable launch after launch, also when a launch is replayed from a graph, and
// whichever of the forms in this file a launch takes (the counters of all of them lie before the
// tagged words of any, see MeetGeom::tagged).
//
// The wait is bounded in time.  A workgroup whose wait runs out (the device is shared with other
// work, so not every workgroup of the block got a place) still produces the right result: for every
// slot of its block that is not published it computes the slice's maximum from memory itself.  That
// is safe even in place, because a workgroup writes its output only after its own wait, which starts
// after it has published; so if the slot is still unpublished after the read, the read saw nothing
// but input.
// ---------------------------------------------------------------------------------------------
constexpr uint32_t kPublished = 0x80000000u;
constexpr uint32_t kMeetGroup = 32;              // workgroups per first-level counter
constexpr uint32_t kMeetHeaderWords = 16;        // words 0..2 as above, the rest of the line unused
constexpr uint32_t kMeetLine = 16;               // 64-bit words of a 128-byte line
constexpr uint32_t kMeetBlocksPerWord = 256;     // blocks counted into one "meetings over" word

struct MeetGeom {
    uint64_t nblocks;
    uint32_t slices;        // workgroups per block
    uint32_t groups;        // first-level counters per block: ceil(slices / kMeetGroup)
    uint32_t stride;        // words from one counter or flag to the next
    uint32_t wait_us;       // how long a workgroup waits for the others before it helps itself
    uint64_t counters, tops, finished;     // first word of each kind of counter
    uint64_t flags, slots;                 // first word of each kind of tagged word; flags == the first tagged word
};

// Zeroes the scratch of a launch whose caller does not keep it between calls.
__global__ void block_sync_clear_kernel(uint64_t* sync, uint64_t words)
{
    const uint64_t i = linear_block() * blockDim.x + threadIdx.x;
    if (i < words) sync[i] = 0ull;
}

// Tag of this launch's meetings; every thread reads it before the workgroup does anything else.  (An
// ordinary load of a wave-uniform address: the word was written by an earlier launch, and this
// launch's only write to it waits for every workgroup to have arrived, that is, to have read it.
// The compiler cannot repeat the load further down, past this kernel's own atomics on the scratch.)
__device__ __forceinline__ uint32_t meet_tag(const uint64_t* scratch)
{
    const uint32_t next = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)scratch[1]) + 1u;
    return next == 0u ? 1u : next;       // (zero is what an unused word holds)
}

// Workgroup s of block b brings the maximum m of its slice and gets the block's maximum back.
// `tag` is meet_tag(); slice_max(i) gives
// each thread's share of the maximum of slice i of the block, from memory.  Called by every thread.
// `ticket` comes back equal to mg.slices - 1 in thread 0 of one workgroup of the block, which then
// knows that every workgroup of the block has arrived: it owes a call of meet_is_over(), for which
// meet_leave() at the end of the kernel is the place (the workgroup's own stores are on their way then).
//
// POLL_SLOTS false: the counters described above (a whole tensor on a thousand workgroups: nobody
// reads more than one flag).  POLL_SLOTS true, for the forms that meet block by block with at most
// a few hundred workgroups per block: a workgroup publishes its slot and the first wavefront polls the
// block's slots until all carry the tag; nothing is waited for but the slots themselves.  The
// block's counter then only counts, after the meeting, who has been there.
template <bool POLL_SLOTS, int THREADS = kThreads, class SliceMax>
__device__ __forceinline__ uint32_t meet_in_block(uint64_t* scratch, const MeetGeom& mg, uint64_t b, uint32_t s, uint32_t tag,
                                                  uint32_t m, uint32_t* lds, uint32_t& shared_word, uint32_t& ticket,
                                                  SliceMax slice_max)
{
    uint64_t* slots = scratch + mg.slots + b * mg.slices;
    ticket = ~0u;
    if (POLL_SLOTS) {
        if (threadIdx.x < 64) {
            const uint64_t mark = ((uint64_t)tag << 32) | kPublished;
            if (threadIdx.x == 0) __hip_atomic_store(&slots[s], mark | m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t start = __builtin_amdgcn_s_memrealtime();          // 100 MHz
            const uint64_t budget = (uint64_t)mg.wait_us * 100u;
            uint32_t acc;
            bool all;
            for (;;) {
                bool ok = true;
                acc = 0u;
                for (uint32_t i = threadIdx.x; i < mg.slices; i += 64u) {
                    const uint64_t a = __hip_atomic_load(&slots[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    ok = ok && (uint32_t)(a >> 32) == tag;
                    const uint32_t mag = (uint32_t)a & ~kPublished;
                    acc = acc > mag ? acc : mag;
                }
                all = __all(ok);
                if (all || __builtin_amdgcn_s_memrealtime() - start >= budget) break;
                __builtin_amdgcn_s_sleep(1);
            }
            acc = wave_max(acc);
            if (threadIdx.x == 0) {
                shared_word = all ? (acc | kPublished) : 0u;
                // been there (and read the epoch long before): counted now, looked at in meet_leave()
                ticket = (uint32_t)__hip_atomic_fetch_add(scratch + mg.counters + b, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    } else if (threadIdx.x == 0) {
        const uint64_t mark = ((uint64_t)tag << 32) | kPublished;
        const uint32_t gi = s / kMeetGroup;
        const uint64_t q = b * mg.groups + gi;
        const uint32_t members = mg.slices - gi * kMeetGroup < kMeetGroup ? mg.slices - gi * kMeetGroup : kMeetGroup;
        uint64_t* counter = scratch + mg.counters + q * mg.stride;
        __hip_atomic_store(&slots[s], mark | m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        uint32_t before = __hip_atomic_fetch_max(reinterpret_cast<uint32_t*>(counter), m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(before) : : "memory");      // slot written, maximum folded in: now count
        const uint64_t r = __hip_atomic_fetch_add(counter, 1ull << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(r >> 32) == members - 1u) {
            // last of the group: everybody's maximum was in before they counted themselves
            uint32_t bm = (uint32_t)r;
            bool last = true;
            __hip_atomic_store(counter, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (mg.groups > 1u) {
                uint64_t* top = scratch + mg.tops + b * mg.stride;
                uint32_t before2 = __hip_atomic_fetch_max(reinterpret_cast<uint32_t*>(top), bm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(before2) : : "memory");
                const uint64_t r2 = __hip_atomic_fetch_add(top, 1ull << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                last = (uint32_t)(r2 >> 32) == mg.groups - 1u;
                bm = (uint32_t)r2;
                if (last) __hip_atomic_store(top, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (last) {
                for (uint32_t i = 0; i < mg.groups; ++i)
                    __hip_atomic_store(&scratch[mg.flags + (b * mg.groups + i) * mg.stride], mark | bm, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                ticket = mg.slices - 1u;
            }
        }
        const uint64_t* flag = scratch + mg.flags + q * mg.stride;
        const uint64_t start = __builtin_amdgcn_s_memrealtime();          // 100 MHz
        const uint64_t budget = (uint64_t)mg.wait_us * 100u;
        uint64_t a = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        while ((uint32_t)(a >> 32) != tag && __builtin_amdgcn_s_memrealtime() - start < budget) {
            __builtin_amdgcn_s_sleep(1);
            a = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        shared_word = (uint32_t)(a >> 32) == tag ? (uint32_t)a : 0u;        // a valid flag has the published bit
    }
    __syncthreads();
    if (shared_word & kPublished) return shared_word & ~kPublished;

    // the wait ran out
    if (threadIdx.x == 0) __hip_atomic_fetch_add(reinterpret_cast<uint32_t*>(scratch), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint32_t bm = 0;
    for (uint32_t i = 0; i < mg.slices; ++i) {
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint64_t a = __hip_atomic_load(&slots[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            shared_word = (uint32_t)(a >> 32) == tag ? (uint32_t)a : 0u;
        }
        __syncthreads();
        uint32_t a = shared_word;
        if (!(a & kPublished)) {
            // the owner of slice i has not published, so it has not written any output yet:
            // read its input; if the slot is still unpublished afterwards, the read was clean
            const uint32_t own = workgroup_max<THREADS>(slice_max(i), lds);
            __syncthreads();
            if (threadIdx.x == 0) {
                const uint64_t again = __hip_atomic_load(&slots[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                shared_word = (uint32_t)(again >> 32) == tag ? (uint32_t)again : 0u;
            }
            __syncthreads();
            a = (shared_word & kPublished) ? shared_word : own;
        }
        a &= ~kPublished;
        bm = bm > a ? bm : a;
    }
    return bm;
}

// The last arrival of block b reports that the block's meeting is over (thread 0 only); the one that
// reports the last block of the launch moves the epoch on, when every workgroup of the launch has
// arrived and therefore read it.
__device__ __forceinline__ void meet_is_over(uint64_t* scratch, const MeetGeom& mg, uint64_t b, uint32_t tag)
{
    bool all = mg.nblocks == 1;
    if (!all) {
        const uint64_t w = b / kMeetBlocksPerWord;
        const uint64_t here = mg.nblocks - w * kMeetBlocksPerWord < kMeetBlocksPerWord ? mg.nblocks - w * kMeetBlocksPerWord
                                                                                         : kMeetBlocksPerWord;
        uint64_t* word = scratch + mg.finished + w;
        if (__hip_atomic_fetch_add(word, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == here - 1u) {
            __hip_atomic_store(word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t words = (mg.nblocks + kMeetBlocksPerWord - 1) / kMeetBlocksPerWord;
            if (__hip_atomic_fetch_add(&scratch[2], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == words - 1u) {
                __hip_atomic_store(&scratch[2], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                all = true;
            }
        }
    }
    if (all) __hip_atomic_store(&scratch[1], (uint64_t)tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// At the end of a kernel: the workgroup that holds the block's last ticket settles the block's account.
template <bool POLL_SLOTS>
__device__ __forceinline__ void meet_leave(uint64_t* scratch, const MeetGeom& mg, uint64_t b, uint32_t tag, uint32_t ticket)
{
    if (threadIdx.x == 0 && ticket == mg.slices - 1u) {
        if (POLL_SLOTS) __hip_atomic_store(scratch + mg.counters + b, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        meet_is_over(scratch, mg, b, tag);
    }
}

// Single pass for contiguous blocks that fit in the register files of the whole chip (for instance
// a 4096 x 4096 tensor quantized as one block).  The grid is small enough for every workgroup to be
// resident at the same time; each loads its slice of 256 * GPT groups into registers, brings the
// slice's maximum to the meeting of its block, and quantizes out of registers: HBM sees each element
// once in and once out.
//
// With 16 groups per thread the kernel must keep to 128 VGPRs (four waves per SIMD, four workgroups
// per CU): that is what lets 1024 workgroups hold a 16 Mi-element tensor.
//
// CLUSTER: the tensor as a whole does not fit, but each block does, and the grid may be far larger
// than the chip.  Workgroups are numbered block by block and dispatched in that order, so the
// workgroups of the lowest unfinished block are always among the resident ones and the grid drains
// block after block; should the dispatcher ever do otherwise, the bounded wait and the exact
// fallback still end every workgroup with the right result.
struct ResidentGeom {
    SliceGeom sg;            // slice_len = 4 * THREADS * GPT elements; slices = workgroups per block
    uint32_t total_wgs;      // nblocks * slices
    MeetGeom meet;
};

template <int MODE, int GPT, bool CLUSTER = false, int THREADS = kThreads>
__global__ __launch_bounds__(THREADS, (GPT >= 16 ? 1024 / THREADS : 1)) void block_resident_kernel(const uint32_t* in, uint32_t* out, uint64_t* scratch,
                                                                  ResidentGeom rg, int wl, int symmetric, RngKey key)
{
    // Stochastic rounding: the random words of the first PRE groups are drawn while the loads are
    // in flight and parked in LDS (36 KiB at most, so four workgroups still share a CU), those of
    // HELD more groups stay in registers; after the wait only the remaining groups pay for Philox,
    // and the arithmetic hides behind the stores.
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? (GPT < 9 ? GPT : 9) : 0;
    constexpr int HELD = MODE == QSIM_STOCHASTIC && GPT >= 16 && !CLUSTER && THREADS == kThreads ? 1 : 0;
    __shared__ uint4 parked[PRE > 0 ? PRE * THREADS : 1];
    __shared__ uint32_t lds[THREADS / 64];
    __shared__ uint32_t shared_word;
    const uint32_t wg = CLUSTER ? (uint32_t)linear_block() : blockIdx.x;
    if (CLUSTER && wg >= rg.total_wgs) return;                   // the whole workgroup leaves together
    const uint32_t b = wg / rg.sg.slices, s = wg - b * rg.sg.slices;
    const uint32_t tag = meet_tag(scratch);
    const SliceView sv = slice_view(rg.sg, b, s);

    // the slice is addressed from a wave-uniform base with small per-thread offsets, which keeps
    // the address arithmetic out of the vector registers that hold the data
    const uint32_t* sin = in + sv.j0 * 4;
    uint32_t* sout = out + sv.j0 * 4;
    const uint64_t slice_end = sv.end - sv.j0 * 4;               // elements reachable from the base
    const int ngroups = (int)sv.groups;
    const bool full = ngroups == THREADS * GPT && slice_end >= 4ull * THREADS * GPT;

    uint4 v[GPT];
    uint32_t m = 0;
    if (full) {
#pragma unroll
        for (int k = 0; k < GPT; ++k) {
            const int t = (int)threadIdx.x + k * THREADS;
            v[k] = to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(sin) + t));
        }
    } else {
#pragma unroll
        for (int k = 0; k < GPT; ++k) {
            const int t = (int)threadIdx.x + k * THREADS;
            v[k] = make_uint4(0u, 0u, 0u, 0u);
            if (t < ngroups) v[k] = load_group<true>(sin, (uint64_t)t, slice_end);
        }
    }
#pragma unroll
    for (int k = 0; k < PRE; ++k) {
        const Words4 r = random_words(sv.j0 + (uint64_t)((int)threadIdx.x + k * THREADS), key, 0u);
        parked[k * THREADS + threadIdx.x] = make_uint4(r.w[0], r.w[1], r.w[2], r.w[3]);
    }
    Words4 held[HELD > 0 ? HELD : 1];
#pragma unroll
    for (int k = 0; k < HELD; ++k) {
        held[k] = random_words(sv.j0 + (uint64_t)((int)threadIdx.x + (PRE + k) * THREADS), key, 0u);
        // (pinned here: left alone, the compiler sinks the computation below the wait to save registers)
        asm volatile("" : "+v"(held[k].w[0]), "+v"(held[k].w[1]), "+v"(held[k].w[2]), "+v"(held[k].w[3]));
    }
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t gm = max4_mag(v[k]);
        m = m > gm ? m : gm;
    }
    m = workgroup_max<THREADS>(m, lds);

    uint32_t ticket;
    const uint32_t bm = meet_in_block<CLUSTER, THREADS>(scratch, rg.meet, b, s, tag, m, lds, shared_word, ticket,
                                               [&](uint32_t i) { return slice_max_frugal(in, slice_view(rg.sg, b, i)); });

    const GridPlan p = block_plan(bm, wl, symmetric);
    const bool finite = wave_plans_are_finite<MODE>(p);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const int t = (int)threadIdx.x + k * THREADS;
        if (full || t < ngroups) {
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) {
                const uint4 w = parked[k * THREADS + threadIdx.x];
                r = Words4{{w.x, w.y, w.z, w.w}};
            } else if (k < PRE + HELD) {
                r = held[k - PRE < 0 ? 0 : k - PRE];
            } else if (MODE == QSIM_STOCHASTIC) {
                r = random_words(sv.j0 + (uint64_t)t, key, 0u);
            }
            const uint4 o = quantize_group_of_block<MODE>(v[k], p, r, finite);
            if (full) __builtin_nontemporal_store(to_u32x4(o), reinterpret_cast<u32x4*>(sout) + t);
            else store_group<true>(sout, (uint64_t)t, slice_end, o);
        }
    }
    meet_leave<CLUSTER>(scratch, rg.meet, b, tag, ticket);
}

// The same block-by-block single pass for blocks along an inner dimension (outer > 1) made of
// aligned segments of at least 64 elements (inner % 4 == 0): per-channel blocks of an
// [N, C, H, W] tensor.  Slice s of block b is elements [s * slice_len, ...) of the block's own
// numbering t = o * inner + i (slice_len = 64 elements per thread: a block of up to 16 Ki elements is
// one workgroup of 256 threads, larger ones are shared by workgroups of 512, two of which fit a CU:
// half as many to meet, [128, 64, 112 x 112] 174.5 us -> 160.1 us); a group's place in the array follows from one division by `inner`
// (multiply-high with a reciprocal rounded up, corrected by at most one) for a thread's first
// group, additions from there.  Up to 512 slices per block (half of the workgroups the chip holds at
// once), which meet as above (counters, flags and epochs packed, one word after the other).
constexpr uint32_t kStridedSliceLen = 4u * kThreads * 16u;
constexpr uint32_t kStridedMaxSlices = 512;

struct StridedClusterGeom {
    uint64_t nblocks;
    uint32_t block_len;      // outer * inner
    uint32_t slice_len;      // 64 elements per thread of the workgroups that share a block: 16 Ki or 32 Ki
    uint32_t slices;         // at most kStridedMaxSlices
    uint32_t inner;          // a multiple of 4, at least 64
    uint32_t magic_inner;    // floor(2^32 / inner) + 1
    uint32_t total_wgs;
    // A thread's groups are 4 * THREADS elements of the block apart.  Counted in groups from the
    // block's first element, the group at element (o, i) sits at o * row_groups + i / 4; from one of a
    // thread's groups to its next that grows by step_groups, and by wrap_groups more when i, having
    // grown by step_rest, passes `inner` (all modulo 2^32: the array has fewer than 2^32 groups).
    uint32_t row_groups;     // nblocks * inner / 4
    uint32_t step_rest;      // (4 * THREADS) % inner
    uint32_t step_groups;    // ((4 * THREADS) / inner) * row_groups + step_rest / 4
    uint32_t wrap_groups;    // row_groups - inner / 4
    MeetGeom meet;
};

// A thread's walk over its groups of a block: `off` is the current group, counted from the block's
// first; two additions and a compare per step instead of a division and a 64-bit product per group.
struct StridedWalk {
    uint32_t i, off;
};

__device__ __forceinline__ StridedWalk strided_walk(const StridedClusterGeom& cg, uint32_t tt)
{
    uint32_t o = __umulhi(tt, cg.magic_inner);           // tt / inner or one more (tt < 2^22)
    uint32_t i = tt - o * cg.inner;
    if ((int32_t)i < 0) {
        o -= 1u;
        i += cg.inner;
    }
    return StridedWalk{i, o * cg.row_groups + i / 4u};
}

__device__ __forceinline__ void strided_step(const StridedClusterGeom& cg, StridedWalk& w)
{
    w.i += cg.step_rest;
    w.off += cg.step_groups;
    if (w.i >= cg.inner) {
        w.i -= cg.inner;
        w.off += cg.wrap_groups;
    }
}

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
    const uint32_t t0 = s * cg.slice_len;
    const uint32_t t1 = (cg.block_len - t0 < cg.slice_len) ? cg.block_len : t0 + cg.slice_len;
    return (t1 - t0) / 4u;
}

template <int MODE, int THREADS>
__global__ __launch_bounds__(THREADS, 1024 / THREADS) void block_cluster_strided_kernel(const uint32_t* in, uint32_t* out, uint64_t* scratch,
                                                                            StridedClusterGeom cg, int wl, int symmetric,
                                                                            RngKey key)
{
    constexpr int GPT = 16;
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? 9 : 0;          // random words parked in LDS, as in the kernel above
    __shared__ uint4 parked[PRE > 0 ? PRE * THREADS : 1];
    __shared__ uint32_t lds[THREADS / 64];
    __shared__ uint32_t shared_word;
    const uint32_t wg = (uint32_t)linear_block();
    if (wg >= cg.total_wgs) return;                                // the whole workgroup leaves together
    const uint32_t b = wg / cg.slices, s = wg - b * cg.slices;
    const uint32_t tag = cg.slices == 1u ? 0u : meet_tag(scratch);
    const uint32_t t0 = s * cg.slice_len;
    const uint32_t ngroups = strided_slice_groups(cg, s);

    const uint64_t jbase = (uint64_t)b * (cg.inner / 4u);           // the block's first group
    StridedWalk walk = strided_walk(cg, t0 + 4u * threadIdx.x);
    uint4 v[GPT];
    uint32_t where[GPT];                                           // kept for the stores
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * THREADS;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        where[k] = walk.off;
        if (t < ngroups) {
            const uint64_t j = jbase + walk.off;
            v[k] = to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(in) + j));
            if (k < PRE) {
                const Words4 r = random_words(j, key, 0u);
                parked[k * THREADS + threadIdx.x] = make_uint4(r.w[0], r.w[1], r.w[2], r.w[3]);
            }
        }
        strided_step(cg, walk);
    }
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t gm = max4_mag(v[k]);
        m = m > gm ? m : gm;
    }
    m = workgroup_max<THREADS>(m, lds);

    // (a block that one workgroup holds alone has nobody to meet and leaves the scratch alone)
    uint32_t ticket = ~0u;
    const uint32_t bm = cg.slices == 1u ? m : meet_in_block<true, THREADS>(scratch, cg.meet, b, s, tag, m, lds, shared_word, ticket, [&](uint32_t i) {
        uint32_t own = 0;
        const uint32_t count = strided_slice_groups(cg, i);
        for (uint32_t t = threadIdx.x; t < count; t += THREADS) {
            const uint4 w = *(reinterpret_cast<const uint4*>(in) + strided_group(cg, b, i * cg.slice_len + 4u * t));
            const uint32_t gm = max4_mag(w);
            own = own > gm ? own : gm;
        }
        return own;
    });

    const GridPlan p = block_plan(bm, wl, symmetric);
    const bool finite = wave_plans_are_finite<MODE>(p);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * THREADS;
        if (t < ngroups) {
            const uint64_t j = jbase + where[k];
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) {
                const uint4 w = parked[k * THREADS + threadIdx.x];
                r = Words4{{w.x, w.y, w.z, w.w}};
            } else if (MODE == QSIM_STOCHASTIC) {
                r = random_words(j, key, 0u);
            }
            __builtin_nontemporal_store(to_u32x4(quantize_group_of_block<MODE>(v[k], p, r, finite)), reinterpret_cast<u32x4*>(out) + j);
        }
    }
    if (cg.slices > 1u) meet_leave<true>(scratch, cg.meet, b, tag, ticket);
}

// The same blocks when one of them fits a single LARGE workgroup (512 or 1024 threads, 16 groups per
// thread: up to 32 Ki or 64 Ki elements): nobody to meet, no scratch; the block's maximum is a
// reduction through LDS.  For the small activation tensors of a network on small images
// ([128, 128, 16, 16] per channel: blocks of 32 Ki elements), where two workgroups of 256 threads
// per block would spend more time finding each other than moving the data.
template <int MODE, int THREADS, int GPT>
__global__ __launch_bounds__(THREADS) void block_strided_wide_kernel(const uint32_t* in, uint32_t* out, StridedClusterGeom cg, int wl,
                                                                     int symmetric, RngKey key)
{
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? (GPT < 9 ? GPT : 9) : 0;   // random words parked in LDS while the loads are in flight
    __shared__ uint4 parked[PRE > 0 ? PRE * THREADS : 1];
    __shared__ uint32_t lds[THREADS / 64];
    const uint32_t b = (uint32_t)linear_block();
    if (b >= cg.nblocks) return;                                   // the whole workgroup leaves together
    const uint32_t ngroups = cg.block_len / 4u;

    const uint64_t jbase = (uint64_t)b * (cg.inner / 4u);           // the block's first group
    StridedWalk walk = strided_walk(cg, 4u * threadIdx.x);
    uint4 v[GPT];
    uint32_t where[GPT];                                           // kept for the stores
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * THREADS;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        where[k] = walk.off;
        if (t < ngroups) {
            const uint64_t j = jbase + walk.off;
            v[k] = to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4*>(in) + j));
            if (k < PRE) {
                const Words4 r = random_words(j, key, 0u);
                parked[k * THREADS + threadIdx.x] = make_uint4(r.w[0], r.w[1], r.w[2], r.w[3]);
            }
        }
        strided_step(cg, walk);
    }
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t gm = max4_mag(v[k]);
        m = m > gm ? m : gm;
    }
    const GridPlan p = block_plan(workgroup_max<THREADS>(m, lds), wl, symmetric);
    const bool finite = wave_plans_are_finite<MODE>(p);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * THREADS;
        if (t < ngroups) {
            const uint64_t j = jbase + where[k];
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) {
                const uint4 w = parked[k * THREADS + threadIdx.x];
                r = Words4{{w.x, w.y, w.z, w.w}};
            } else if (MODE == QSIM_STOCHASTIC) {
                r = random_words(j, key, 0u);
            }
            __builtin_nontemporal_store(to_u32x4(quantize_group_of_block<MODE>(v[k], p, r, finite)), reinterpret_cast<u32x4*>(out) + j);
        }
    }
}

// The same for segments of any length from 64 elements at any alignment (inner % 4 != 0, or arrays
// that are only dword aligned): per-channel blocks of an [N, C, 27, 27] tensor, and long contiguous
// blocks (outer == 1, one segment each) of odd length.  The unit is still
// a group of the ARRAY's numbering (elements 4j .. 4j + 3), so that one Philox block serves it;
// a segment starting at element S is covered by groups S / 4 ... (S + inner - 1) / 4, of which the
// first and the last may hold elements of a neighbouring block ("strangers": loaded, because one
// dwordx4 load at a dword-aligned address is still the cheapest, then masked out of the maximum and
// never stored).  Every segment is given G = (inner + 2) / 4 + 1 group slots, the most it can
// cover; slot t of a block is slot u = t % G of segment o = t / G, unused when that segment covers
// fewer groups.  The slots of a block are dealt out evenly to its slices, at most 16 per thread:
// 4096 each for workgroups of 256 threads, 8192 for workgroups of 512 (THREADS; two of those share
// a CU where four of the smaller do: half as many workgroups have to meet per block).
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
    // A thread's slots are one workgroup's threads apart: from one to its next, u grows by step_rest and the
    // segment's first element by step_elems, and by row_elems more when u passes G.
    uint32_t row_elems;      // nblocks * inner: from a segment of a block to its next (0 for a contiguous block)
    uint32_t threads;        // of a workgroup: 256, or 512 when a block has more slots than 256 threads hold
    uint32_t step_rest;      // threads % G
    uint32_t step_elems;     // (threads / G) * row_elems
    MeetGeom meet;
};

constexpr uint32_t kRaggedSliceGroups = kThreads * 16u;

// Slot t of block b: the group j it stands for and which of its four elements belong to the block
// (bit e of `mask`; 0 for an unused slot).
__device__ __forceinline__ void ragged_slot(const RaggedClusterGeom& cg, uint32_t b, uint32_t t, uint64_t& j, uint32_t& mask)
{
    uint32_t o = 0u, u = t;
    if (cg.block_groups != cg.seg_groups) {               // (uniform; a contiguous block is one segment)
        o = __umulhi(t, cg.magic_groups);                 // t / G or one more (t < 2^20)
        u = t - o * cg.seg_groups;
        if ((int32_t)u < 0) {
            o -= 1u;
            u += cg.seg_groups;
        }
    }
    const uint64_t start = ((uint64_t)o * cg.nblocks + b) * cg.inner;      // first element of the segment
    const uint32_t r = (uint32_t)start & 3u;
    j = (start >> 2) + u;
    // (the last of contiguous blocks may be short)
    const uint32_t len = start + cg.inner > cg.n ? (uint32_t)(cg.n - start) : cg.inner;
    // the segment is elements [lo, hi) of the group's own numbering
    const int32_t lo = (int32_t)r - 4 * (int32_t)u, hi = (int32_t)(len + r) - 4 * (int32_t)u;
    const uint32_t below_hi = hi >= 4 ? 0xFu : hi <= 0 ? 0u : (1u << hi) - 1u;
    const uint32_t from_lo = lo <= 0 ? 0xFu : (0xFu << lo) & 0xFu;
    mask = below_hi & from_lo;
}

// Which elements of slot u of a segment belong to it, when the segment is elements [r, r + len) of
// the numbering that starts at its first group: bits max(lo, 0) .. min(hi, 4) - 1.
__device__ __forceinline__ uint32_t ragged_mask(uint32_t r, uint32_t u, uint32_t len)
{
    const int32_t lo = (int32_t)r - 4 * (int32_t)u, hi = (int32_t)(len + r) - 4 * (int32_t)u;      // lo < hi
    const int32_t l = lo < 0 ? 0 : (lo > 4 ? 4 : lo), h = hi < 0 ? 0 : (hi > 4 ? 4 : hi);
    return ((1u << (h - l)) - 1u) << l;
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

template <int MODE, int THREADS>
__global__ __launch_bounds__(THREADS, 1024 / THREADS) void block_cluster_ragged_kernel(const uint32_t* in, uint32_t* out, uint64_t* scratch,
                                                                           RaggedClusterGeom cg, int wl, int symmetric,
                                                                           RngKey key)
{
    constexpr int GPT = 16;
    constexpr int PRE = MODE == QSIM_STOCHASTIC ? 9 : 0;          // random words parked in LDS, as in the kernels above
    __shared__ uint4 parked[PRE > 0 ? PRE * THREADS : 1];
    __shared__ uint32_t lds[THREADS / 64];
    __shared__ uint32_t shared_word;
    const uint32_t wg = (uint32_t)linear_block();
    if (wg >= cg.total_wgs) return;                                // the whole workgroup leaves together
    const uint32_t b = wg / cg.slices, s = wg - b * cg.slices;
    const uint32_t tag = cg.slices == 1u ? 0u : meet_tag(scratch);
    const uint32_t t0 = s * cg.slice_groups;
    const uint32_t nslots = ragged_slice_slots(cg, s);
    const bool short_tail = (cg.n & 3u) != 0u;                     // the array's last group is not whole

    // The block's first segment starts at element sbase = 4 * jbase + e0; a later segment starts
    // `rel` elements further on.  (Only the last of contiguous blocks may be short.)
    const uint64_t sbase = (uint64_t)b * cg.inner;
    const uint64_t jbase = sbase >> 2;
    const uint32_t e0 = (uint32_t)sbase & 3u;
    const uint32_t len = cg.block_groups == cg.seg_groups && sbase + cg.inner > cg.n ? (uint32_t)(cg.n - sbase) : cg.inner;
    uint32_t o = 0u, u = t0 + threadIdx.x;                         // the thread's first slot: slot u of segment o
    if (cg.block_groups != cg.seg_groups) {                        // (uniform; a contiguous block is one segment)
        o = __umulhi(u, cg.magic_groups);                          // u / G or one more (u < 2^20)
        u -= o * cg.seg_groups;
        if ((int32_t)u < 0) {
            o -= 1u;
            u += cg.seg_groups;
        }
    }
    uint32_t rel = o * cg.row_elems;

    // Every load is one unconditional dwordx4 inside the array, so that all sixteen are in flight
    // together: an unused slot reads the group before it, and the array's short last group reads
    // the array's last four elements instead (put right below, `shift` elements further on).
    uint4 v[GPT];
    uint32_t where[GPT];                                           // group of each slot, counted from jbase: kept for the stores
    uint32_t shifts = 0u;
    uint32_t masks[2] = {0u, 0u};                                  // four bits per group
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * THREADS;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        const uint32_t e = e0 + rel;
        where[k] = (e >> 2) + u;
        if (t < nslots) {
            const uint32_t mask = ragged_mask(e & 3u, u, len);
            masks[k / 8] |= mask << (4 * (k % 8));
            const uint64_t j = jbase + where[k];
            const uint32_t* src = in + 4u * j;
            if (mask == 0u) src -= 4;
            if (short_tail) {
                const uint64_t at = (uint64_t)(src - in);
                if (at + 4u > cg.n) {
                    if (mask != 0u) shifts |= (uint32_t)(at + 4u - cg.n) << (2 * k);      // 1..3
                    src = in + (cg.n - 4u);
                }
            }
            v[k] = to_uint4(__builtin_nontemporal_load(reinterpret_cast<const u32x4_at_dword*>(src)));
            if (k < PRE) {
                const Words4 r = random_words(j, key, 0u);
                parked[k * THREADS + threadIdx.x] = make_uint4(r.w[0], r.w[1], r.w[2], r.w[3]);
            }
        }
        u += cg.step_rest;
        rel += cg.step_elems;
        if (u >= cg.seg_groups) {
            u -= cg.seg_groups;
            rel += cg.row_elems;
        }
    }
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t mask = (masks[k / 8] >> (4 * (k % 8))) & 0xFu;
        if (short_tail) {
            const uint32_t sh = (shifts >> (2 * k)) & 3u;          // element e of the group was loaded as word e + sh
            if (sh == 1u) v[k] = make_uint4(v[k].y, v[k].z, v[k].w, 0u);
            else if (sh == 2u) v[k] = make_uint4(v[k].z, v[k].w, 0u, 0u);
            else if (sh == 3u) v[k] = make_uint4(v[k].w, 0u, 0u, 0u);
        }
        const uint32_t gm = max4_mag(keep_masked(v[k], mask));       // strangers stay in v[k]: quantized below, never stored
        m = m > gm ? m : gm;
    }
    m = workgroup_max<THREADS>(m, lds);

    uint32_t ticket = ~0u;
    const uint32_t bm = cg.slices == 1u ? m : meet_in_block<true, THREADS>(scratch, cg.meet, b, s, tag, m, lds, shared_word, ticket, [&](uint32_t i) {
        // slice i of this block from memory, element by element where a group is shared
        uint32_t own = 0;
        const uint32_t count = ragged_slice_slots(cg, i);
        for (uint32_t t = threadIdx.x; t < count; t += THREADS) {
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
    const bool finite = wave_plans_are_finite<MODE>(p);
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * THREADS;
        if (t < nslots) {
            const uint64_t j = jbase + where[k];
            const uint32_t mask = (masks[k / 8] >> (4 * (k % 8))) & 0xFu;
            Words4 r = {{0u, 0u, 0u, 0u}};
            if (k < PRE) {
                const uint4 w = parked[k * THREADS + threadIdx.x];
                r = Words4{{w.x, w.y, w.z, w.w}};
            } else if (MODE == QSIM_STOCHASTIC) {
                r = random_words(j, key, 0u);
            }
            const uint4 q = quantize_group_of_block<MODE>(v[k], p, r, finite);
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
    if (cg.slices > 1u) meet_leave<true>(scratch, cg.meet, b, tag, ticket);
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
            const bool finite = wave_plans_are_finite<MODE>(p);
            __builtin_nontemporal_store(to_u32x4(quantize_group_of_block<MODE>(v[k], p, r, finite)), reinterpret_cast<u32x4*>(out) + where[k]);
        }
    }
}

}  // namespace qsim
