// Block floating point in a single pass for blocks larger than one workgroup: the workgroups hold
// the data in registers and meet over their maxima (whole tensor, block by block for contiguous rows
// and for blocks along an inner dimension), and several short strided blocks per workgroup.
#pragma once

#include "qsim_kernel_common.hpp"
#include "qsim_block_two_pass_kernels.hpp"

namespace qsim {

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
// that are only dword aligned): per-channel blocks of an [N, C, 27, 27] tensor, and long contiguous
// blocks (outer == 1, one segment each) of odd length.  The unit is still
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
    uint32_t masks[2] = {0u, 0u};                                  // four bits per group
#pragma unroll
    for (int k = 0; k < GPT; ++k) {
        const uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        v[k] = make_uint4(0u, 0u, 0u, 0u);
        if (t < nslots) {
            uint64_t j;
            uint32_t mask;
            ragged_slot(cg, b, t0 + t, j, mask);
            masks[k / 8] |= mask << (4 * (k % 8));
            uint64_t at = 4u * j;
            if (mask == 0u) at -= 4u;
            if (at + 4u > cg.n) {
                if (mask != 0u) shifts |= (uint32_t)(at + 4u - cg.n) << (2 * k);      // 1..3
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
        // (the group number is worked out again rather than kept: sixteen of them do not fit the
        // registers next to sixteen groups; the empty asm keeps the compiler from finding out that it
        // is the same computation)
        uint32_t t = threadIdx.x + (uint32_t)k * kThreads;
        asm volatile("" : "+v"(t));
        if (t < nslots) {
            uint64_t j;
            uint32_t unused;
            ragged_slot(cg, b, t0 + t, j, unused);
            const uint32_t mask = (masks[k / 8] >> (4 * (k % 8))) & 0xFu;
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

}  // namespace qsim
