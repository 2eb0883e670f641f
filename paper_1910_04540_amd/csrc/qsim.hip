// libqsim: the C-ABI entry points (include/qsim.h).  Each validates its arguments on the host,
// resolves the format into a device plan, picks the kernel variant and enqueues it on the caller's
// stream.  No entry point allocates device memory, and none synchronises except
// qsim_sgd_table_build, which waits for its own copy of the table.
#include <hip/hip_runtime.h>

#include <atomic>
#include <vector>

#include "qsim.h"
#include "qsim_device.hpp"
#include "qsim_host.hpp"
#include "qsim_kernels.hpp"

namespace qsim {

// The caller's stream.  Called once by every entry point, after validation and before its first
// launch: an error that an earlier, unrelated HIP call of the caller left pending is dropped here,
// so that launch_status() reports this call's launches only.
static hipStream_t as_stream(void* s)
{
    (void)hipGetLastError();
    return reinterpret_cast<hipStream_t>(s);
}
static int launch_status() { return hipGetLastError() == hipSuccess ? QSIM_OK : QSIM_ERR_LAUNCH; }
static RngKey make_key(uint64_t seed, uint32_t stream_id, uint64_t index0)
{
    return RngKey{(uint32_t)seed, (uint32_t)(seed >> 32), stream_id, index0 / 4};
}
static const uint32_t* u32(const float* p) { return reinterpret_cast<const uint32_t*>(p); }
static uint32_t* u32(float* p) { return reinterpret_cast<uint32_t*>(p); }

// Grid of `blocks` workgroups folded over x and y (see linear_block()); blocks <= kGridX * 65535.
static dim3 folded(uint64_t blocks)
{
    if (blocks <= kGridX) return dim3((unsigned)blocks);
    return dim3(kGridX, (unsigned)((blocks + kGridX - 1) / kGridX));
}
// The same over x and z, with y given (see linear_block_xz()).
static dim3 folded_xz(uint64_t blocks, unsigned y)
{
    if (blocks <= kGridX) return dim3((unsigned)blocks, y);
    return dim3(kGridX, y, (unsigned)((blocks + kGridX - 1) / kGridX));
}

// Groups per thread of the elementwise kernels.
constexpr int kUnroll = 1;

// ---- elementwise ---------------------------------------------------------------------------
template <class Op, int MODE>
static int launch_elementwise_mode(const float* in, float* out, uint64_t n, const Op& op, const RngKey& key,
                                   hipStream_t stream)
{
    const uint64_t groups = (n + 3) / 4;
    const uint64_t blocks = (groups + kStreamThreads * kUnroll - 1) / (kStreamThreads * kUnroll);
    hipLaunchKernelGGL((elementwise_kernel<Op, MODE, kUnroll>), folded(blocks), dim3(kStreamThreads), 0, stream,
                       u32(in), u32(out), n, groups, op, key);
    return launch_status();
}

template <class Op>
static int launch_elementwise(const float* in, float* out, uint64_t n, int rounding, const Op& op, const RngKey& key,
                              hipStream_t stream)
{
    switch (rounding) {
    case QSIM_RN_EVEN: return launch_elementwise_mode<Op, QSIM_RN_EVEN>(in, out, n, op, key, stream);
    case QSIM_RN_AWAY: return launch_elementwise_mode<Op, QSIM_RN_AWAY>(in, out, n, op, key, stream);
    case QSIM_RN_ZERO: return launch_elementwise_mode<Op, QSIM_RN_ZERO>(in, out, n, op, key, stream);
    default:           return launch_elementwise_mode<Op, QSIM_STOCHASTIC>(in, out, n, op, key, stream);
    }
}

// Unaligned arrays: dword accesses, format resolved at run time.
static int launch_elementwise_rt(const float* in, float* out, uint64_t n, const FormatPlan& f, const RngKey& key,
                                 hipStream_t stream)
{
    const uint64_t groups = (n + 3) / 4;
    const uint64_t blocks = (groups + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(elementwise_rt_kernel, folded(blocks), dim3(kThreads), 0, stream, u32(in), u32(out), n,
                       groups, f, key);
    return launch_status();
}

// ---- block floating point ------------------------------------------------------------------
// How a block-quantize call may be carried out: every form the shape admits, decided on the host
// from the shape alone, so that qsim_block_workspace_bytes and qsim_block_quantize always agree.
// Which of them runs also depends on the alignment of the arrays and on the device; the scratch is
// sized for the largest.
struct BlockSchedule {
    bool one_launch;       // contiguous blocks small enough for one team or workgroup each
    SliceGeom sg;          // otherwise: two launches over slices
    bool cluster;          // many contiguous blocks of up to 512 register-resident slices each: single pass per block
    bool strided_packed;   // outer > 1, whole-group segments, blocks of at most 2048 elements: several per workgroup
    StridedPackedGeom spg;
    bool ragged_runs;      // the same for segments of any length and alignment (the arrays' own groups, shared edge groups)
    int ragged_runs_gpt;   // groups per thread: 8, or 16 when a block needs that many
    RaggedRunsGeom rrg;
    bool strided_cluster;  // outer > 1, aligned segments of >= 64 elements, blocks of up to 512 slices: the same
    StridedClusterGeom scg;
    bool strided_ragged;   // outer > 1, segments of >= 64 elements of any length and alignment: the same
    RaggedClusterGeom rcg;
    bool flat;             // outer > 1 and short rows: the flat form (any alignment)
    FlatGeom fg;
    bool column;           // outer > 1 and short blocks: the column form (any row length, any alignment)
    ColumnGeom cg;
    // The scratch has two parts, so that a caller may keep it between calls (QSIM_WORKSPACE_KEPT):
    // the words of the single-pass forms' meetings come first, and only the meetings write there;
    // the partial maxima of the two-pass forms start at `partial_offset`.
    uint64_t sync_counters; // 64-bit words of header and counters of the single-pass forms the shape may take: the largest
    uint64_t sync_tagged;  // the same for their tagged words, which start behind sync_counters in every form
    size_t sync_bytes;     // (sync_counters + sync_tagged) * 8
    size_t partial_bytes;  // the largest scratch of its two-pass forms
    size_t partial_offset; // sync_bytes rounded up to 256
    size_t workspace;      // partial_offset + partial_bytes
};

constexpr uint64_t kCachedMaxInner = 16384;      // 256 threads x 16 groups x 4 elements
constexpr int kWideThreads = 1024;
constexpr uint64_t kWideCachedMaxInner = 65536;  // 1024 threads x 16 groups x 4 elements
constexpr uint64_t kClusterSliceLen = 4ull * kThreads * 16;     // 16 groups per thread
constexpr uint64_t kClusterMaxSlices = 512;      // half of the workgroups the chip holds at once
constexpr uint64_t kClusterMaxWgs = 1ull << 22;
constexpr uint32_t kMaxSlices = 1024;
constexpr uint64_t kMinSliceLen = 16384;
constexpr uint64_t kTileLen = 4ull * kTileGroups;
constexpr uint32_t kMaxResidentWgs = 4096;       // bound of the single-pass form's scratch
constexpr uint32_t kMaxResidentGroups = 128;     // counters (and blocks) of one resident launch: a line each
constexpr uint64_t kPackedSmallTensor = 1ull << 23;   // elements; see block_schedule
constexpr uint64_t kRaggedMinGroups = 2048;      // smallest block, in group slots, for the single pass over odd segments
constexpr uint64_t kCachedTensorElements = 96ull << 20;   // 384 MiB: see column_geometry
constexpr uint64_t kColumnThreads = 1ull << 19;  // threads the column form aims for
constexpr uint64_t kColumnShortInner = 64;       // below: always; up to kColumnMaxInner: when there are enough blocks
constexpr uint64_t kColumnMaxInner = 4096;       // to keep the one-wavefront-per-block fold parallel
constexpr uint64_t kColumnManyBlocks = 1024;      // (a quarter of both also qualifies: 256 blocks of up to 1024)
constexpr uint32_t kColumnParts = 8;             // slices left after the first, coalesced fold of its column maxima
constexpr uint64_t kFlatWorkgroups = 1024;       // workgroups of the flat form (four per CU)
constexpr uint64_t kMultiTiles = 1ull << 30;     // tiles of one multi-tensor launch (running counts are 32-bit)

// Row slices of the column form: a thread owns a run of four columns.
static ColumnGeom column_geometry(uint64_t outer, uint64_t nblocks, uint64_t inner)
{
    ColumnGeom cg;
    cg.outer = outer;
    cg.row = (uint32_t)(nblocks * inner);
    cg.row_groups = (uint32_t)(((uint64_t)cg.row + 3) / 4);
    const uint64_t columns = cg.row_groups;
    cg.inner = (uint32_t)inner;
    cg.nblocks = (uint32_t)nblocks;
    // enough threads to fill the chip, at least 16 rows per thread when there are that many
    uint64_t slices = (kColumnThreads + columns - 1) / columns;
    const uint64_t most = (outer + 15) / 16;
    if (slices > most) slices = most;
    if (slices > 65535) slices = 65535;
    cg.rows_per_slice = (uint32_t)((outer + slices - 1) / slices);
    cg.slices = (uint32_t)((outer + cg.rows_per_slice - 1) / cg.rows_per_slice);
    // Pass 2 finds a tensor of up to 256 MiB or so in the memory-side cache when pass 1 has read it
    // with ordinary loads (64 Mi elements: 138 us against 144 us with non-temporal loads in pass 1;
    // 16 Mi: 38 us against 47 us); a larger one does not stay, and streaming it is faster
    // (128 Mi elements: 271 us against 289 us).
    cg.stream_first = outer * cg.row > kCachedTensorElements ? 1u : 0u;
    return cg;
}

// Scratch of a column form: column maxima of every slice, the same folded to kColumnParts slices, block maxima.
static size_t column_bytes(const ColumnGeom& cg)
{
    const size_t fewer = cg.slices > 2 * kColumnParts ? kColumnParts : 0;      // only many slices are folded twice
    return ((size_t)cg.slices + fewer) * (size_t)cg.row_groups * 4 * sizeof(uint32_t) + (size_t)cg.nblocks * sizeof(uint32_t);
}

static std::atomic<uint32_t> g_barrier_wait_us{2000u};

// Words of the meetings of `nblocks` blocks of `slices` workgroups each (see meet_in_block): the
// counters right behind the header, the tagged words from `tagged` on, which is the same for every
// form a shape may take, so that no form ever leaves a tagged word where another has a counter.
struct MeetLayout {
    MeetGeom geom;
    uint64_t counter_words;   // header and counters
    uint64_t tagged_words;    // flags and slots
};

static MeetLayout meet_layout(uint64_t nblocks, uint32_t slices, uint32_t stride, bool poll_slots, uint64_t tagged = 0)
{
    MeetLayout l;
    MeetGeom& g = l.geom;
    g.nblocks = nblocks;
    g.slices = slices;
    g.groups = poll_slots ? 1u : (slices + kMeetGroup - 1) / kMeetGroup;
    g.stride = stride;
    g.wait_us = g_barrier_wait_us.load(std::memory_order_relaxed);
    g.counters = kMeetHeaderWords;
    g.tops = g.counters + nblocks * g.groups * stride;
    g.finished = g.tops + (poll_slots ? 0 : nblocks * stride);
    l.counter_words = g.finished + (nblocks + kMeetBlocksPerWord - 1) / kMeetBlocksPerWord;
    g.flags = tagged ? tagged : l.counter_words;
    const uint64_t flag_words = poll_slots ? 0 : nblocks * g.groups * stride;
    g.slots = g.flags + flag_words;
    l.tagged_words = flag_words + nblocks * slices;
    return l;
}

// The resident form gives every counter and flag a line of its own while they are few; its scratch is at most this.
constexpr uint64_t kResidentCounterWords = kMeetHeaderWords + 2ull * kMaxResidentGroups * kMeetLine + 1;
constexpr uint64_t kResidentTaggedWords = (uint64_t)kMaxResidentGroups * kMeetLine + kMaxResidentWgs;

// Zeroes what a launch with this layout reads of a scratch that its caller does not keep.
static void clear_scratch(uint64_t* scratch, const MeetLayout& l, hipStream_t stream)
{
    const uint64_t words = l.geom.flags + l.tagged_words;
    hipLaunchKernelGGL(block_sync_clear_kernel, folded((words + kThreads - 1) / kThreads), dim3(kThreads), 0, stream, scratch, words);
}

// How a block's slots are dealt out to workgroups of `threads` threads, 16 slots per thread (see RaggedClusterGeom).
static void ragged_workgroups(RaggedClusterGeom& cg, uint32_t threads)
{
    const uint32_t per_wg = threads * 16u;
    cg.threads = threads;
    cg.slices = (cg.block_groups + per_wg - 1u) / per_wg;
    cg.slice_groups = (cg.block_groups + cg.slices - 1u) / cg.slices;
    cg.total_wgs = (uint32_t)(cg.nblocks * cg.slices);
    cg.step_rest = threads % cg.seg_groups;
    cg.step_elems = (threads / cg.seg_groups) * cg.row_elems;
}

// The walk of a thread over its groups when the workgroup has `threads` threads (see StridedClusterGeom).
static void strided_steps(StridedClusterGeom& cg, uint32_t threads)
{
    const uint32_t step = 4u * threads;
    cg.step_rest = step % cg.inner;
    cg.step_groups = (uint32_t)((uint64_t)(step / cg.inner) * cg.row_groups + cg.step_rest / 4u);      // modulo 2^32
}

static BlockSchedule block_schedule(uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner)
{
    BlockSchedule s;
    memset(&s, 0, sizeof(s));
    if (nblocks == 1 && outer > 1) {      // one block is one block, however the view splits it
        inner = n;
        outer = 1;
    }
    s.sg.g = BlockGeom{n, outer, nblocks, inner};
    s.sg.block_len = outer * inner;
    s.one_launch = outer == 1 && inner <= kCachedMaxInner;
    if (s.one_launch) return s;
    uint64_t slices = (s.sg.block_len + kMinSliceLen - 1) / kMinSliceLen;
    if (slices > kMaxSlices) slices = kMaxSlices;
    uint64_t slice_len = (s.sg.block_len + slices - 1) / slices;
    slice_len = (slice_len + kTileLen - 1) / kTileLen * kTileLen;
    slices = (s.sg.block_len + slice_len - 1) / slice_len;
    s.sg.slice_len = slice_len;
    s.sg.slices = (uint32_t)slices;
    auto sync_needs = [&s](uint64_t counter_words, uint64_t tagged_words) {
        if (s.sync_counters < counter_words) s.sync_counters = counter_words;
        if (s.sync_tagged < tagged_words) s.sync_tagged = tagged_words;
    };
    auto meeting = [&](uint32_t slices_each) {
        const MeetLayout l = meet_layout(nblocks, slices_each, 1, true);
        sync_needs(l.counter_words, l.tagged_words);
    };
    auto partial_needs = [&s](size_t bytes) {
        if (s.partial_bytes < bytes) s.partial_bytes = bytes;
    };
    partial_needs((size_t)(nblocks * slices * sizeof(uint32_t)));
    // the single-pass form over resident workgroups
    if (outer == 1) sync_needs(kResidentCounterWords, kResidentTaggedWords);
    // the same kernel meeting block by block (the scratch is sized for workgroups of 16,384 elements;
    // the launch uses half as many of 32,768)
    const uint64_t cluster_slices = (inner + kClusterSliceLen - 1) / kClusterSliceLen;
    if (outer == 1 && inner > kWideCachedMaxInner && cluster_slices <= kClusterMaxSlices &&
        nblocks * cluster_slices <= kClusterMaxWgs) {
        s.cluster = true;
        meeting((uint32_t)cluster_slices);
    }
    // (the runs a workgroup reads are 16 KiB / outer long: only for few outer indices, or for a
    // tensor small enough that one launch instead of three or four outweighs the scattered reads:
    // [128, 512, 4, 4] per channel 14.4 us -> 8.9 us, [128, 4096, 16] 21.6 us -> 18.7 us)
    if (outer > 1 && (outer <= 16 || n <= kPackedSmallTensor) && inner % 4 == 0 && s.sg.block_len <= 2048) {
        s.strided_packed = true;
        s.spg.nblocks = nblocks;
        s.spg.outer_inner = (uint32_t)s.sg.block_len;
        s.spg.groups_per_block = s.spg.outer_inner / 4;
        s.spg.magic_groups = s.spg.groups_per_block > 1 ? (uint32_t)((1ull << 32) / s.spg.groups_per_block) + 1u : 0u;
        s.spg.inner = (uint32_t)inner;
        s.spg.magic_inner = (uint32_t)((1ull << 32) / inner) + 1u;
        s.spg.blocks_per_wg = 1024u / s.spg.groups_per_block;
    }
    // (these two forms count groups and elements from a block's start in 32 bits)
    if (outer > 1 && (outer <= 16 || n <= kPackedSmallTensor) && s.sg.block_len <= 2048) {
        // every run of a workgroup gets (rows * inner + 6) / 4 + 1 group slots; as many blocks as 2048
        // slots hold, or 4096 when not even one fits
        for (int gpt = 8; gpt <= 16 && !s.ragged_runs; gpt *= 2) {
            const uint64_t per_run = (uint64_t)kThreads * gpt / outer;            // slots a run may take
            if (per_run < 3) continue;
            uint64_t rows = (4 * (per_run - 1) - 6) / inner;                       // (rows * inner + 6) / 4 + 1 <= per_run
            if (rows * inner > 65535) rows = 65535 / inner;
            if (rows > (uint64_t)kRaggedMaxRows) rows = kRaggedMaxRows;
            if (rows > nblocks) rows = nblocks;
            if (rows * inner < 64) continue;            // (runs of a few elements: the forms that walk the tensor front to back do better)
            // a small tensor is spread over at least 1024 workgroups, as long as the runs keep 64 elements
            const uint64_t fewest = (63 + inner) / inner, spread = nblocks / 1024 > fewest ? nblocks / 1024 : fewest;
            if (rows > spread) rows = spread;
            s.ragged_runs = true;
            s.ragged_runs_gpt = gpt;
            s.rrg.n = n;
            s.rrg.nblocks = nblocks;
            s.rrg.outer = (uint32_t)outer;
            s.rrg.inner = (uint32_t)inner;
            s.rrg.rows_per_wg = (uint32_t)rows;
            s.rrg.run_slots = (uint32_t)((rows * inner + 6) / 4 + 1);
            s.rrg.magic_slots = (uint32_t)((1ull << 32) / s.rrg.run_slots) + 1u;
            s.rrg.magic_inner = inner > 1 ? (uint32_t)((1ull << 32) / inner) + 1u : 0u;
        }
    }
    if (outer > 1 && inner % 4 == 0 && inner >= 64 && inner <= (1ull << 23) && n < (1ull << 34) &&
        s.sg.block_len <= (uint64_t)kStridedMaxSlices * kStridedSliceLen) {
        // a block that one workgroup of 256 threads holds keeps that workgroup; larger blocks are shared
        // by workgroups of 512 threads, 32 Ki elements each
        const uint64_t slice_len = s.sg.block_len <= kStridedSliceLen ? kStridedSliceLen : 2 * kStridedSliceLen;
        const uint64_t slices_each = (s.sg.block_len + slice_len - 1) / slice_len;
        if (nblocks * slices_each <= kClusterMaxWgs) {
            s.strided_cluster = true;
            s.scg.nblocks = nblocks;
            s.scg.block_len = (uint32_t)s.sg.block_len;
            s.scg.slice_len = (uint32_t)slice_len;
            s.scg.slices = (uint32_t)slices_each;
            s.scg.inner = (uint32_t)inner;
            s.scg.magic_inner = (uint32_t)((1ull << 32) / inner) + 1u;
            s.scg.total_wgs = (uint32_t)(nblocks * slices_each);
            s.scg.row_groups = (uint32_t)(nblocks * inner / 4);
            s.scg.wrap_groups = s.scg.row_groups - (uint32_t)(inner / 4);
            strided_steps(s.scg, (uint32_t)(slice_len / 64));
            meeting(s.scg.slices);
        }
    }
    if (inner >= 64 && inner <= (1ull << 23) && n < (1ull << 32)) {          // (contiguous blocks too: one segment each)
        const uint64_t seg_groups = (inner + 2) / 4 + 1;
        const unsigned __int128 block_groups = (unsigned __int128)outer * seg_groups;
        // (a block has workgroups of its own, four of which fit a CU: with fewer than eight loads per
        // thread in flight they do not keep the memory busy, and the column form measured faster)
        if (block_groups >= kRaggedMinGroups && block_groups <= (uint64_t)kStridedMaxSlices * kRaggedSliceGroups) {
            // (sized for workgroups of 256 threads; the launch may share a block among half as many of 512)
            const uint64_t slices_each = ((uint64_t)block_groups + kRaggedSliceGroups - 1) / kRaggedSliceGroups;
            if (nblocks * slices_each <= kClusterMaxWgs) {
                s.strided_ragged = true;
                s.rcg.n = n;
                s.rcg.nblocks = nblocks;
                s.rcg.inner = (uint32_t)inner;
                s.rcg.seg_groups = (uint32_t)seg_groups;
                s.rcg.magic_groups = (uint32_t)((1ull << 32) / seg_groups) + 1u;
                s.rcg.block_groups = (uint32_t)block_groups;
                s.rcg.row_elems = outer > 1 ? (uint32_t)(nblocks * inner) : 0u;
                ragged_workgroups(s.rcg, kThreads);
                meeting(s.rcg.slices);
            }
        }
    }
    // the flat form: short rows, few enough blocks for a table in LDS
    const unsigned __int128 row128 = (unsigned __int128)nblocks * inner;
    if (outer > 1 && row128 <= kFlatMaxRow && nblocks <= (uint64_t)kFlatMaxBlocks) {
        s.flat = true;
        FlatGeom& fg = s.fg;
        fg.n = n;
        fg.groups = (n + 3) / 4;
        fg.row = (uint32_t)row128;
        fg.inner = (uint32_t)inner;
        fg.nblocks = (uint32_t)nblocks;
        fg.magic_row = fg.row > 1 ? (uint32_t)((1ull << 32) / fg.row) + 1u : 0u;
        fg.magic_inner = fg.inner > 1 ? (uint32_t)((1ull << 32) / fg.inner) + 1u : 0u;
        const uint64_t steps = (fg.groups + kFlatStepGroups - 1) / kFlatStepGroups;
        const uint64_t wgs = steps < kFlatWorkgroups ? steps : kFlatWorkgroups;
        fg.groups_per_wg = (steps + wgs - 1) / wgs * kFlatStepGroups;
        fg.wgs = (uint32_t)((fg.groups + fg.groups_per_wg - 1) / fg.groups_per_wg);
        fg.stream_first = n > kCachedTensorElements ? 1u : 0u;
        fg.copies = 1;
        while (fg.copies < 64 && 2 * fg.copies * ((fg.nblocks + 3u) & ~3u) <= (uint32_t)kFlatMaxBlocks) fg.copies *= 2;
        partial_needs((size_t)(kFlatWorkgroups + 1) * nblocks * sizeof(uint32_t));
    }
    // the column form: short segments (a thread walking down a column jumps a whole row per step, which
    // only pays when the alternative would do a division per run of a short segment), and segments of
    // up to 4096 elements when there are many blocks (the alternative gives every block a workgroup
    // of its own, however small the block; the fold here is one wavefront per block over
    // slices * inner values, so it needs many blocks to be parallel).  Rows short enough for 32-bit
    // column arithmetic.
    const unsigned __int128 row = (unsigned __int128)nblocks * inner;
    if (outer > 1 && row <= (1ull << 31) && outer <= (1ull << 32) &&
        (inner < kColumnShortInner || (inner <= kColumnMaxInner / 4 && nblocks >= kColumnManyBlocks / 4) ||
         (inner <= kColumnMaxInner && nblocks >= kColumnManyBlocks))) {
        s.column = true;
        s.cg = column_geometry(outer, nblocks, inner);
        partial_needs(column_bytes(s.cg));
    }
    s.sync_bytes = (size_t)((s.sync_counters + s.sync_tagged) * sizeof(uint64_t));
    s.partial_offset = (s.sync_bytes + 255) & ~(size_t)255;
    s.workspace = s.partial_offset + s.partial_bytes;
    return s;
}

// ---- single pass over resident workgroups ----------------------------------------------------

// Workgroups of block_resident_kernel<MODE, GPT> that are certain to be resident together on the
// current device: four per CU at most.  At that occupancy every resource is accounted for by
// construction (128 VGPRs by launch bounds, about 100 SGPRs, 36 KiB of LDS each); the runtime's
// occupancy query is only allowed to lower the figure, because it has been seen to ignore the
// scalar register file.
constexpr int kResidentPerCu = 4;

template <int MODE, int GPT, int THREADS = kThreads>
static uint32_t resident_capacity()
{
    static std::atomic<int> cache[64];          // per device; 0 = not known yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int c = cache[dev].load(std::memory_order_relaxed);
    if (c == 0) {
        int per_cu = 0, cus = 0;
        const bool ok =
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)block_resident_kernel<MODE, GPT, false, THREADS>,
                                                         THREADS, 0) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess;
        // (a query that fails, say in a state of the runtime that does not allow it, is asked again by the
        // next call: this one takes the two-pass form)
        if (!ok || per_cu <= 0 || cus <= 0) {
            (void)hipGetLastError();
            return 0u;
        }
        if (per_cu > kResidentPerCu * kThreads / THREADS) per_cu = kResidentPerCu * kThreads / THREADS;
        c = per_cu * cus;
        cache[dev].store(c, std::memory_order_relaxed);
    }
    return (uint32_t)c;
}

// Tries the single-pass form with GPT groups per thread; false = does not fit (nothing launched).
// The launch is an ordinary one: the grid is no larger than what the device holds at once, and a
// workgroup that waits in vain (the device is shared with other work) falls back to an exact slow
// path, so residency is a matter of speed, not of correctness or termination.
template <int MODE, int GPT, int THREADS = kThreads>
static bool try_resident(const uint32_t* in, uint32_t* out, const BlockGeom& g, int wl, int symmetric, const RngKey& key,
                         uint64_t* scratch, uint64_t tagged, bool kept, hipStream_t stream)
{
    const uint64_t slice_len = 4ull * THREADS * GPT;
    const uint64_t slices = (g.inner + slice_len - 1) / slice_len;
    const uint64_t total = slices * g.nblocks;
    if (total > kMaxResidentWgs || total > resident_capacity<MODE, GPT, THREADS>()) return false;
    // a line for every counter, flag and epoch while they are few; packed otherwise (many small blocks)
    const uint64_t groups = g.nblocks * ((slices + kMeetGroup - 1) / kMeetGroup);
    const MeetLayout meet = meet_layout(g.nblocks, (uint32_t)slices, groups <= kMaxResidentGroups ? kMeetLine : 1u, false, tagged);
    if (meet.counter_words > kResidentCounterWords || meet.tagged_words > kResidentTaggedWords) return false;
    ResidentGeom rg;
    rg.sg.g = g;
    rg.sg.block_len = g.inner;
    rg.sg.slice_len = slice_len;
    rg.sg.slices = (uint32_t)slices;
    rg.total_wgs = (uint32_t)total;
    rg.meet = meet.geom;
    if (!kept) clear_scratch(scratch, meet, stream);
    hipLaunchKernelGGL((block_resident_kernel<MODE, GPT, false, THREADS>), dim3((unsigned)total), dim3(THREADS), 0, stream, in, out,
                       scratch, rg, wl, symmetric, key);
    return true;
}

// The single-pass form block by block, for more blocks than the chip holds at once (see the kernel).
template <int MODE>
static bool try_cluster(const uint32_t* in, uint32_t* out, const BlockGeom& g, int wl, int symmetric, const RngKey& key,
                        uint64_t* scratch, uint64_t tagged, bool kept, hipStream_t stream)
{
    // workgroups of 512 threads, 32 Ki elements each: half as many to meet as with 256 threads
    // (64 rows of 1 Mi elements 107 us -> 97 us)
    const uint64_t slice_len = 2 * kClusterSliceLen;
    const uint64_t slices = (g.inner + slice_len - 1) / slice_len;
    if (resident_capacity<MODE, 16>() < kClusterMaxSlices) return false;     // a block's workgroups must fit together
    const MeetLayout meet = meet_layout(g.nblocks, (uint32_t)slices, 1u, true, tagged);
    ResidentGeom rg;
    rg.sg.g = g;
    rg.sg.block_len = g.inner;
    rg.sg.slice_len = slice_len;
    rg.sg.slices = (uint32_t)slices;
    rg.total_wgs = (uint32_t)(slices * g.nblocks);
    rg.meet = meet.geom;
    if (!kept) clear_scratch(scratch, meet, stream);
    hipLaunchKernelGGL((block_resident_kernel<MODE, 16, true, 2 * kThreads>), folded(rg.total_wgs), dim3(2 * kThreads), 0, stream, in,
                       out, scratch, rg, wl, symmetric, key);
    return true;
}

template <int MODE>
static bool try_resident_any(const uint32_t* in, uint32_t* out, const BlockGeom& g, int wl, int symmetric, const RngKey& key,
                             uint64_t* scratch, uint64_t tagged, bool kept, hipStream_t stream)
{
    // fewest groups per thread that still fit: more workgroups in flight hide more latency
    return try_resident<MODE, 1>(in, out, g, wl, symmetric, key, scratch, tagged, kept, stream) ||
           try_resident<MODE, 2>(in, out, g, wl, symmetric, key, scratch, tagged, kept, stream) ||
           try_resident<MODE, 4>(in, out, g, wl, symmetric, key, scratch, tagged, kept, stream) ||
           try_resident<MODE, 8>(in, out, g, wl, symmetric, key, scratch, tagged, kept, stream) ||
           try_resident<MODE, 16>(in, out, g, wl, symmetric, key, scratch, tagged, kept, stream);
}

template <int MODE, int GPT, bool WHOLE>
static void launch_block_cached(const uint32_t* in, uint32_t* out, const BlockGeom& g, int team_log2, int wl, int symmetric,
                                const RngKey& key, hipStream_t stream)
{
    // Teams live inside a wavefront and share nothing beyond it.  One wavefront per workgroup streams
    // best when every lane of every team has work (block lengths 4, 8, ..., 1024: 80 % -> 84 % of
    // peak); with idle lanes the 256-thread workgroup measured faster (rows of 100 or 1000 elements).
    if constexpr (!WHOLE) {
        const uint64_t groups = (g.inner + 3) / 4;
        if ((groups & (groups - 1)) == 0) {
            const uint64_t per_wg = (uint64_t)(kStreamThreads >> team_log2);
            hipLaunchKernelGGL((block_cached_kernel<MODE, GPT, false, kStreamThreads>), folded((g.nblocks + per_wg - 1) / per_wg),
                               dim3(kStreamThreads), 0, stream, in, out, g, team_log2, wl, symmetric, key);
            return;
        }
    }
    const uint64_t teams_per_wg = WHOLE ? 1 : (uint64_t)(kThreads >> team_log2);
    const uint64_t blocks = (g.nblocks + teams_per_wg - 1) / teams_per_wg;
    hipLaunchKernelGGL((block_cached_kernel<MODE, GPT, WHOLE>), folded(blocks), dim3(kThreads), 0, stream, in, out, g,
                       team_log2, wl, symmetric, key);
}

template <int MODE, int GPT>
static void launch_block_ragged(const uint32_t* in, uint32_t* out, const BlockGeom& g, bool wide, int wl, int symmetric,
                                const RngKey& key, hipStream_t stream)
{
    // whole blocks per workgroup: their elements plus the strangers in the first and last group fit the registers
    uint64_t rows = (4ull * kThreads * GPT - 6) / g.inner;
    if (rows > (uint64_t)kRaggedMaxRows) rows = kRaggedMaxRows;
    const uint32_t magic = g.inner > 1 ? (uint32_t)((1ull << 32) / g.inner) + 1u : 0u;
    const uint64_t blocks = (g.nblocks + rows - 1) / rows;
    if (wide)
        hipLaunchKernelGGL((block_ragged_kernel<MODE, GPT, true>), folded(blocks), dim3(kThreads), 0, stream, in, out, g,
                           (uint32_t)rows, magic, wl, symmetric, key);
    else
        hipLaunchKernelGGL((block_ragged_kernel<MODE, GPT, false>), folded(blocks), dim3(kThreads), 0, stream, in, out, g,
                           (uint32_t)rows, magic, wl, symmetric, key);
}

template <int MODE>
static void launch_block_cluster_ragged(const uint32_t* in, uint32_t* out, const RaggedClusterGeom& geom, int wl, int symmetric,
                                        const RngKey& key, uint64_t* scratch, uint64_t tagged, bool kept, hipStream_t stream)
{
    RaggedClusterGeom cg = geom;
    // A block of more slots than 256 threads hold is shared by workgroups of 512 threads, half as many
    // to meet ([128, 64, 55 x 55] nearest 45.3 us -> 43.6 us); not with stochastic rounding, whose
    // arithmetic wants four independent workgroups per CU (47.9 us -> 50.2 us with two).
    if (MODE != QSIM_STOCHASTIC && cg.block_groups > kRaggedSliceGroups) ragged_workgroups(cg, 2 * kThreads);
    const MeetLayout meet = meet_layout(cg.nblocks, cg.slices, 1u, true, tagged);
    cg.meet = meet.geom;
    if (!kept && cg.slices > 1u) clear_scratch(scratch, meet, stream);       // (one workgroup per block: nothing meets)
    if (cg.threads == (uint32_t)kThreads)
        hipLaunchKernelGGL((block_cluster_ragged_kernel<MODE, kThreads>), folded(cg.total_wgs), dim3(kThreads), 0, stream, in, out,
                           scratch, cg, wl, symmetric, key);
    else
        hipLaunchKernelGGL((block_cluster_ragged_kernel<MODE, 2 * kThreads>), folded(cg.total_wgs), dim3(2 * kThreads), 0, stream, in,
                           out, scratch, cg, wl, symmetric, key);
}

template <int MODE>
static int launch_block_mode(const float* in, float* out, const BlockSchedule& s, int wl, int symmetric,
                             const RngKey& key, void* workspace, bool kept, hipStream_t stream)
{
    const uint32_t* pin = u32(in);
    uint32_t* pout = u32(out);
    const BlockGeom& g = s.sg.g;
    // whole groups per block: every block starts on a group boundary (a single block always does)
    const bool vec = aligned16(in) && aligned16(out) && (g.inner % 4 == 0 || g.nblocks == 1);
    if (s.one_launch) {
        const uint64_t groups = (g.inner + 3) / 4;
        if (vec && groups <= 256) {
            // a team of 1..64 lanes per block, up to four groups per lane
            int team_log2 = 0;
            while (team_log2 < 6 && (1ull << team_log2) < groups) ++team_log2;
            const uint64_t per_lane = (groups + (1ull << team_log2) - 1) >> team_log2;
            if (per_lane <= 1) launch_block_cached<MODE, 1, false>(pin, pout, g, team_log2, wl, symmetric, key, stream);
            else if (per_lane <= 2) launch_block_cached<MODE, 2, false>(pin, pout, g, team_log2, wl, symmetric, key, stream);
            else launch_block_cached<MODE, 4, false>(pin, pout, g, team_log2, wl, symmetric, key, stream);
        } else if (vec && groups <= 256 * 16) {
            const uint64_t per_lane = (groups + kThreads - 1) / kThreads;
            if (per_lane <= 2) launch_block_cached<MODE, 2, true>(pin, pout, g, 8, wl, symmetric, key, stream);
            else if (per_lane <= 4) launch_block_cached<MODE, 4, true>(pin, pout, g, 8, wl, symmetric, key, stream);
            else if (per_lane <= 8) launch_block_cached<MODE, 8, true>(pin, pout, g, 8, wl, symmetric, key, stream);
            else launch_block_cached<MODE, 16, true>(pin, pout, g, 8, wl, symmetric, key, stream);
        } else if (g.inner + 6 <= 4ull * kThreads * 16) {
            // any block length, aligned arrays or not: whole blocks per workgroup, the tensor's own groups
            const bool wide = aligned16(in) && aligned16(out);
            if (g.inner + 6 <= 4ull * kThreads * 4) launch_block_ragged<MODE, 4>(pin, pout, g, wide, wl, symmetric, key, stream);
            else if (g.inner + 6 <= 4ull * kThreads * 8) launch_block_ragged<MODE, 8>(pin, pout, g, wide, wl, symmetric, key, stream);
            else launch_block_ragged<MODE, 16>(pin, pout, g, wide, wl, symmetric, key, stream);
        } else {
            hipLaunchKernelGGL((block_rows_kernel<MODE>), folded(g.nblocks), dim3(kThreads), 0, stream, pin,
                               pout, g, wl, symmetric, key);
        }
        return launch_status();
    }
    // meetings of the single-pass forms at the start of the scratch, partial maxima of the others behind them
    uint64_t* scratch = reinterpret_cast<uint64_t*>(workspace);
    uint32_t* partial = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(workspace) + s.partial_offset);
    const dim3 grid = folded_xz(g.nblocks, s.sg.slices);
    // Segments of at most 128 elements that do not start and end on 64-byte lines: a kernel that
    // works block by block writes their first and last lines in two parts at different times, and
    // the forms that walk the tensor front to back (flat, column) measured faster, two passes and all
    // ([7048, 62, 76] 92 us -> 72 us, [8000, 32, 128] one element off 94 us -> 74 us).
    const bool short_segments = g.inner <= 128 && (s.flat || s.column);
    if (vec && g.outer == 1) {
        // single pass when the blocks fit in the chip's registers, else the streaming two-pass form:
        // blocks on grid.y (folded when there are more than 65535), slices on grid.x
        if (try_resident_any<MODE>(pin, pout, g, wl, symmetric, key, scratch, s.sync_counters, kept, stream)) return launch_status();
        if (g.inner <= kWideCachedMaxInner) {
            // too many blocks to hold at once, but each fits the registers of one large workgroup, 16
            // groups per lane: two workgroups of 512 threads per CU, or one of 1024
            if (g.inner <= kWideCachedMaxInner / 2)
                hipLaunchKernelGGL((block_cached_kernel<MODE, 16, true, kWideThreads / 2>), folded(g.nblocks),
                                   dim3(kWideThreads / 2), 0, stream, pin, pout, g, 9, wl, symmetric, key);
            else
                hipLaunchKernelGGL((block_cached_kernel<MODE, 16, true, kWideThreads>), folded(g.nblocks), dim3(kWideThreads), 0,
                                   stream, pin, pout, g, 10, wl, symmetric, key);
            return launch_status();
        }
        if (s.cluster && try_cluster<MODE>(pin, pout, g, wl, symmetric, key, scratch, s.sync_counters, kept, stream)) return launch_status();
        const unsigned by = (unsigned)(g.nblocks < 65535 ? g.nblocks : 65535);
        hipLaunchKernelGGL(block_slice_max_kernel, dim3(s.sg.slices, by), dim3(kThreads), 0, stream, pin, partial, s.sg);
        hipLaunchKernelGGL((block_slice_apply_kernel<MODE>), dim3(s.sg.slices, by), dim3(kThreads), 0, stream, pin, pout,
                           partial, s.sg.slices, s.sg, wl, symmetric, key);
    } else if (g.outer == 1 && s.strided_ragged && resident_capacity<MODE, 16>() >= kStridedMaxSlices) {
        // contiguous blocks of up to 8 Mi elements whose length is not a multiple of four, or in
        // arrays that are only dword aligned: single pass, block by block, over the array's own groups
        launch_block_cluster_ragged<MODE>(pin, pout, s.rcg, wl, symmetric, key, scratch, s.sync_counters, kept, stream);
    } else if (vec && s.strided_packed) {
        const uint64_t wgs = (g.nblocks + s.spg.blocks_per_wg - 1) / s.spg.blocks_per_wg;
        hipLaunchKernelGGL((block_strided_packed_kernel<MODE>), folded(wgs), dim3(kThreads), 0, stream, pin, pout, s.spg, wl,
                           symmetric, key);
    } else if (s.ragged_runs) {
        // the same for segments that are not whole groups, or in arrays that are only dword aligned
        const uint64_t wgs = (g.nblocks + s.rrg.rows_per_wg - 1) / s.rrg.rows_per_wg;
        if (s.ragged_runs_gpt == 8)
            hipLaunchKernelGGL((block_ragged_runs_kernel<MODE, 8>), folded(wgs), dim3(kThreads), 0, stream, pin, pout, s.rrg, wl,
                               symmetric, key);
        else
            hipLaunchKernelGGL((block_ragged_runs_kernel<MODE, 16>), folded(wgs), dim3(kThreads), 0, stream, pin, pout, s.rrg, wl,
                               symmetric, key);
    } else if (vec && s.strided_cluster && !(short_segments && g.inner % 16 != 0) &&
               resident_capacity<MODE, 16>() >= kStridedMaxSlices) {
        // single pass, block by block (see the kernel): the workgroups of a block must fit together
        StridedClusterGeom cg = s.scg;
        // two to four workgroups per block: one large workgroup holds it alone, with nobody to meet
        // (not with stochastic rounding when blocks of more than 32 Ki elements are fewer than the
        // CUs: sixteen Philox blocks per thread on a quarter of the chip then take longer than a
        // meeting does; 64 blocks of 64 Ki elements 17.2 us against 11.9 us)
        const bool few_large = MODE == QSIM_STOCHASTIC && cg.block_len > 4u * 512u * 16u && cg.nblocks < 256;
        if (cg.slices > 1u && cg.block_len <= 4u * 1024u * 16u && !few_large) {
            strided_steps(cg, cg.block_len <= 4u * 512u * 16u ? 512u : 1024u);
            if (cg.block_len <= 4u * 512u * 16u)
                hipLaunchKernelGGL((block_strided_wide_kernel<MODE, 512, 16>), folded(cg.nblocks), dim3(512), 0, stream, pin, pout, cg, wl,
                                   symmetric, key);
            else
                hipLaunchKernelGGL((block_strided_wide_kernel<MODE, 1024, 16>), folded(cg.nblocks), dim3(1024), 0, stream, pin, pout, cg,
                                   wl, symmetric, key);
            return launch_status();
        }
        const MeetLayout meet = meet_layout(cg.nblocks, cg.slices, 1u, true, s.sync_counters);
        cg.meet = meet.geom;
        if (!kept && cg.slices > 1u) clear_scratch(scratch, meet, stream);   // (one workgroup per block: nothing meets)
        if (cg.slice_len == kStridedSliceLen) {
            hipLaunchKernelGGL((block_cluster_strided_kernel<MODE, kThreads>), folded(cg.total_wgs), dim3(kThreads), 0, stream, pin,
                               pout, scratch, cg, wl, symmetric, key);
        } else {
            strided_steps(cg, 2 * kThreads);
            hipLaunchKernelGGL((block_cluster_strided_kernel<MODE, 2 * kThreads>), folded(cg.total_wgs), dim3(2 * kThreads), 0, stream,
                               pin, pout, scratch, cg, wl, symmetric, key);
        }
    } else if (s.strided_ragged && !short_segments && resident_capacity<MODE, 16>() >= kStridedMaxSlices) {
        // the same for segments of any length and alignment
        launch_block_cluster_ragged<MODE>(pin, pout, s.rcg, wl, symmetric, key, scratch, s.sync_counters, kept, stream);
    } else if (s.flat && !(vec && g.inner > 128) &&
               (!s.column || g.nblocks < 64 || s.fg.row < 2048 || g.nblocks * 8192 <= g.n)) {
        // short rows, unless long aligned segments stream well through the slice kernels: always when
        // the column form cannot run; otherwise where that form is weak (few blocks make its fold
        // serial, short rows give it few threads per row), and wherever the per-workgroup tables of
        // block maxima (1024 x nblocks words, written and read once) are small next to the tensor
        // ([11910, 145, 19] 93 us -> 67 us, [8192, 1024, 4] 79 us -> 67 us; [4096, 4096, 1], whose
        // tables are a quarter of the tensor, stays with the column form: 38 us against 49 us)
        const FlatGeom& fg = s.fg;
        uint32_t* blockmax = partial + (size_t)kFlatWorkgroups * fg.nblocks;
        hipLaunchKernelGGL(block_flat_max_kernel, dim3(fg.wgs), dim3(kThreads), 0, stream, pin, partial, blockmax, fg);
        hipLaunchKernelGGL(block_fold_rows_once_kernel, dim3((fg.nblocks + 31u) / 32u, (fg.wgs + kFoldOnceRows - 1u) / kFoldOnceRows),
                           dim3(kThreads), 0, stream, partial, blockmax, fg.nblocks, fg.wgs);
        hipLaunchKernelGGL((block_flat_apply_kernel<MODE>), dim3(fg.wgs), dim3(kThreads), 0, stream, pin, pout, blockmax, fg, wl,
                           symmetric, key);
    } else if (s.column) {
        // dwordx4 accesses at group boundaries when rows are whole groups and the arrays aligned, at any dword otherwise
        const ColumnGeom& cg = s.cg;
        const bool wide = cg.row % 4 == 0 && aligned16(in) && aligned16(out);
        const size_t row_words = (size_t)cg.row_groups * 4;
        uint32_t* fewer = partial + (size_t)cg.slices * row_words;
        uint32_t* blockmax = fewer + (cg.slices > 2 * kColumnParts ? (size_t)kColumnParts * row_words : 0);
        const dim3 cgrid((cg.row_groups + kThreads - 1) / kThreads, cg.slices);
        uint4* colmax = reinterpret_cast<uint4*>(partial);
        if (wide) hipLaunchKernelGGL(block_column_max_kernel<true>, cgrid, dim3(kThreads), 0, stream, pin, colmax, cg);
        else hipLaunchKernelGGL(block_column_max_kernel<false>, cgrid, dim3(kThreads), 0, stream, pin, colmax, cg);
        // fold: over slices first when there are many (neighbouring threads on neighbouring columns),
        // then one wavefront per block, or one thread per block when a block has few values left
        ColumnGeom rest = cg;
        const uint32_t* folded_from = partial;
        if (cg.slices > 2 * kColumnParts) {
            rest.slices = kColumnParts;
            folded_from = fewer;
            hipLaunchKernelGGL(block_fold_rows_kernel, dim3((unsigned)((row_words + kThreads - 1) / kThreads), kColumnParts),
                               dim3(kThreads), 0, stream, partial, fewer, (uint32_t)row_words, cg.slices, kColumnParts);
        }
        // blocks of one column: the few rows of column maxima that are left are folded by pass 2 itself
        const uint32_t parts = cg.inner == 1 ? rest.slices : 0u;
        const uint4* colparts = reinterpret_cast<const uint4*>(folded_from);
        if (parts == 0u && (uint64_t)rest.slices * rest.inner <= 64)
            hipLaunchKernelGGL(block_column_fold_small_kernel, folded((cg.nblocks + kThreads - 1) / kThreads), dim3(kThreads), 0,
                               stream, folded_from, blockmax, rest);
        else if (parts == 0u)
            hipLaunchKernelGGL(block_column_fold_kernel, folded((cg.nblocks + kThreads / 64 - 1) / (kThreads / 64)),
                               dim3(kThreads), 0, stream, folded_from, blockmax, rest);
        if (wide)
            hipLaunchKernelGGL((block_column_apply_kernel<MODE, true>), cgrid, dim3(kThreads), 0, stream, pin, pout, blockmax,
                               colparts, parts, cg, wl, symmetric, key);
        else if (MODE != QSIM_STOCHASTIC)
            hipLaunchKernelGGL((block_column_apply_kernel<MODE, false>), cgrid, dim3(kThreads), 0, stream, pin, pout, blockmax,
                               colparts, parts, cg, wl, symmetric, key);
        else {
            // (63 runs per wavefront: see the kernel)
            const uint32_t runs_per_wg = kColumnSharedRuns * (kThreads / 64);
            const dim3 shared_grid((cg.row_groups + runs_per_wg - 1) / runs_per_wg, cg.slices);
            hipLaunchKernelGGL((block_column_apply_kernel<MODE, false>), shared_grid, dim3(kThreads), 0, stream, pin, pout,
                               blockmax, colparts, parts, cg, wl, symmetric, key);
        }
    } else if (vec) {
        hipLaunchKernelGGL((block_partial_max_kernel<true>), grid, dim3(kThreads), 0, stream, pin, partial, s.sg);
        hipLaunchKernelGGL((block_apply_kernel<MODE, true>), grid, dim3(kThreads), 0, stream, pin, pout, partial, s.sg.slices,
                           s.sg, wl, symmetric, key);
    } else {
        hipLaunchKernelGGL((block_partial_max_kernel<false>), grid, dim3(kThreads), 0, stream, pin, partial, s.sg);
        hipLaunchKernelGGL((block_apply_kernel<MODE, false>), grid, dim3(kThreads), 0, stream, pin, pout, partial, s.sg.slices,
                           s.sg, wl, symmetric, key);
    }
    return launch_status();
}

// Slices of the two-pass form for any shape: the schedule's, or one slice per block for the small
// contiguous blocks the schedule handles in one launch.
static SliceGeom two_pass_geometry(const BlockSchedule& s)
{
    SliceGeom sg = s.sg;
    if (s.one_launch) {
        sg.slices = 1;
        sg.slice_len = (sg.block_len + kTileLen - 1) / kTileLen * kTileLen;
    }
    return sg;
}

template <int MODE>
static int launch_block_given_max(const float* in, float* out, const SliceGeom& sg, int wl, int symmetric, const RngKey& key,
                                  const uint32_t* block_max, hipStream_t stream)
{
    const dim3 grid = folded_xz(sg.g.nblocks, sg.slices);
    const bool vec = aligned16(in) && aligned16(out) && (sg.g.inner % 4 == 0 || sg.g.nblocks == 1);
    if (vec && sg.g.outer == 1) {
        // contiguous blocks: the streaming form (blocks on grid.y, folded when there are more than 65535)
        const unsigned by = (unsigned)(sg.g.nblocks < 65535 ? sg.g.nblocks : 65535);
        hipLaunchKernelGGL((block_slice_apply_kernel<MODE>), dim3(sg.slices, by), dim3(kThreads), 0, stream, u32(in), u32(out),
                           block_max, 1u, sg, wl, symmetric, key);
    } else if (vec)
        hipLaunchKernelGGL((block_apply_kernel<MODE, true>), grid, dim3(kThreads), 0, stream, u32(in), u32(out), block_max, 1u,
                           sg, wl, symmetric, key);
    else
        hipLaunchKernelGGL((block_apply_kernel<MODE, false>), grid, dim3(kThreads), 0, stream, u32(in), u32(out), block_max,
                           1u, sg, wl, symmetric, key);
    return launch_status();
}

}  // namespace qsim

using namespace qsim;

extern "C" {

int qsim_float_quantize(const float* in, float* out, uint64_t n, int exp_bits, int man_bits, int rounding,
                        uint32_t flags, uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    return qsim_float_quantize_at(in, out, n, 0, exp_bits, man_bits, rounding, flags, seed, stream_id, hip_stream);
}

int qsim_float_quantize_at(const float* in, float* out, uint64_t n, uint64_t index0, int exp_bits, int man_bits,
                           int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    if (!valid_rounding(rounding)) return QSIM_ERR_ROUNDING;
    if (!valid_float(exp_bits, man_bits) || !valid_flags(flags)) return QSIM_ERR_FORMAT;
    if (n > kMaxElements || !valid_index0(index0)) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!in || !out) return QSIM_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_ERR_OVERLAP;
    const qsim_format fmt{1, exp_bits, man_bits, rounding, flags};
    FormatPlan f;
    const int status = make_format_plan(&fmt, &f);
    if (status != QSIM_OK) return status;
    const RngKey key = make_key(seed, stream_id, index0);
    hipStream_t stream = as_stream(hip_stream);
    if (!aligned16(in) || !aligned16(out)) return launch_elementwise_rt(in, out, n, f, key, stream);
    if (f.float_form == kFloatGeneral) return launch_elementwise(in, out, n, rounding, FloatGeneralOp{f.flt}, key, stream);
    if (f.flt.denormal_inputs) return launch_elementwise(in, out, n, rounding, FloatShiftOp<true>{f.flt}, key, stream);
    return launch_elementwise(in, out, n, rounding, FloatShiftOp<false>{f.flt}, key, stream);
}

int qsim_fixed_quantize(const float* in, float* out, uint64_t n, int wl, int fl, int rounding, uint32_t flags,
                        uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    return qsim_fixed_quantize_at(in, out, n, 0, wl, fl, rounding, flags, seed, stream_id, hip_stream);
}

int qsim_fixed_quantize_at(const float* in, float* out, uint64_t n, uint64_t index0, int wl, int fl, int rounding,
                           uint32_t flags, uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    if (!valid_rounding(rounding)) return QSIM_ERR_ROUNDING;
    if (!valid_fixed(wl, fl) || !valid_flags(flags)) return QSIM_ERR_FORMAT;
    if (n > kMaxElements || !valid_index0(index0)) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!in || !out) return QSIM_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_ERR_OVERLAP;
    const qsim_format fmt{2, wl, fl, rounding, flags};
    FormatPlan f;
    const int status = make_format_plan(&fmt, &f);
    if (status != QSIM_OK) return status;
    const RngKey key = make_key(seed, stream_id, index0);
    hipStream_t stream = as_stream(hip_stream);
    if (!aligned16(in) || !aligned16(out)) return launch_elementwise_rt(in, out, n, f, key, stream);
    return launch_elementwise(in, out, n, rounding, FixedOp{f.grid}, key, stream);
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
    return qsim_block_quantize_at(in, out, n, outer, nblocks, inner, 0, wl, rounding, flags, seed, stream_id, workspace,
                                  workspace_bytes, hip_stream);
}

// Everything of qsim_block_quantize_at after the validation that does not depend on whose the scratch is.
static int block_quantize_checked(const float* in, float* out, uint64_t n, const BlockSchedule& s, uint64_t index0, int wl,
                                  int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id, void* workspace,
                                  hipStream_t stream)
{
    const RngKey key = make_key(seed, stream_id, index0);
    const int symmetric = (flags & QSIM_SYMMETRIC) ? 1 : 0;
    const bool kept = (flags & QSIM_WORKSPACE_KEPT) != 0;
    (void)n;
    switch (rounding) {
    case QSIM_RN_EVEN: return launch_block_mode<QSIM_RN_EVEN>(in, out, s, wl, symmetric, key, workspace, kept, stream);
    case QSIM_RN_AWAY: return launch_block_mode<QSIM_RN_AWAY>(in, out, s, wl, symmetric, key, workspace, kept, stream);
    case QSIM_RN_ZERO: return launch_block_mode<QSIM_RN_ZERO>(in, out, s, wl, symmetric, key, workspace, kept, stream);
    default:           return launch_block_mode<QSIM_STOCHASTIC>(in, out, s, wl, symmetric, key, workspace, kept, stream);
    }
}

// Validation of a block-quantize call up to (not including) the scratch.
static int check_block_call(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner,
                            uint64_t index0, int wl, int rounding, uint32_t flags)
{
    if (!valid_rounding(rounding)) return QSIM_ERR_ROUNDING;
    if (!valid_block_wl(wl) || !valid_block_flags(flags)) return QSIM_ERR_FORMAT;
    if (n > kMaxElements || !valid_index0(index0)) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!valid_block_shape(n, outer, nblocks, inner)) return QSIM_ERR_SHAPE;
    if (!in || !out) return QSIM_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_ERR_OVERLAP;
    if (nblocks > 0x7fffffffull) return QSIM_ERR_UNSUPPORTED;
    return QSIM_OK;
}

int qsim_block_quantize_at(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner,
                           uint64_t index0, int wl, int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id,
                           void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const int status = check_block_call(in, out, n, outer, nblocks, inner, index0, wl, rounding, flags);
    if (status != QSIM_OK || n == 0) return status;
    const BlockSchedule s = block_schedule(n, outer, nblocks, inner);
    if (s.workspace) {
        if (!workspace || !aligned16(workspace) || workspace_bytes < s.workspace) return QSIM_ERR_WORKSPACE;
        if (ranges_overlap(workspace, s.workspace, in, n * 4) || ranges_overlap(workspace, s.workspace, out, n * 4))
            return QSIM_ERR_OVERLAP;
    }
    return block_quantize_checked(in, out, n, s, index0, wl, rounding, flags, seed, stream_id, workspace, as_stream(hip_stream));
}

// Scratch of qsim_block_quantize_static: one array per GPU, held from load to exit.  In host code the
// array's name is only a handle for the runtime; its address on a device comes from
// hipGetSymbolAddress with that device current, once per device, and only that address is used.
static __device__ __align__(256) unsigned char scratch[QSIM_STATIC_SCRATCH_BYTES];

static void* static_scratch()
{
    static std::atomic<void*> address[64];      // per device; NULL = not looked up yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    void* p = address[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        address[dev].store(p, std::memory_order_release);
    }
    return p;
}

int qsim_block_quantize_static(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner,
                               int wl, int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    if (flags & QSIM_WORKSPACE_KEPT) return QSIM_ERR_FORMAT;      // the array is shared by every shape: always cleared
    const int status = check_block_call(in, out, n, outer, nblocks, inner, 0, wl, rounding, flags);
    if (status != QSIM_OK || n == 0) return status;
    const BlockSchedule s = block_schedule(n, outer, nblocks, inner);
    if (s.workspace > (size_t)QSIM_STATIC_SCRATCH_BYTES) return QSIM_ERR_WORKSPACE;
    void* workspace = nullptr;
    if (s.workspace) {
        workspace = static_scratch();
        if (!workspace) return QSIM_ERR_LAUNCH;
    }
    return block_quantize_checked(in, out, n, s, 0, wl, rounding, flags, seed, stream_id, workspace, as_stream(hip_stream));
}

int qsim_block_max(const float* in, uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner, uint32_t* block_max,
                   void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (n == 0 || n > kMaxElements || !valid_block_shape(n, outer, nblocks, inner)) return QSIM_ERR_SHAPE;
    if (!in || !block_max) return QSIM_ERR_NULL;
    if (nblocks > 0x7fffffffull) return QSIM_ERR_UNSUPPORTED;
    if (ranges_overlap(block_max, nblocks * sizeof(uint32_t), in, n * 4)) return QSIM_ERR_OVERLAP;
    const BlockSchedule s = block_schedule(n, outer, nblocks, inner);
    const SliceGeom sg = two_pass_geometry(s);
    uint32_t* partial = block_max;                       // one slice per block: pass 1 writes the result itself
    if (sg.slices > 1) {
        // (behind the words a kept scratch holds for qsim_block_quantize, like every two-pass form)
        const size_t need = s.partial_offset + (size_t)nblocks * sg.slices * sizeof(uint32_t);
        if (!workspace || !aligned16(workspace) || workspace_bytes < need) return QSIM_ERR_WORKSPACE;
        if (ranges_overlap(workspace, need, in, n * 4) || ranges_overlap(workspace, need, block_max, nblocks * sizeof(uint32_t)))
            return QSIM_ERR_OVERLAP;
        partial = reinterpret_cast<uint32_t*>(static_cast<unsigned char*>(workspace) + s.partial_offset);
    }
    hipStream_t stream = as_stream(hip_stream);
    const dim3 grid = folded_xz(nblocks, sg.slices);
    const bool vec = aligned16(in) && (sg.g.inner % 4 == 0 || sg.g.nblocks == 1);
    if (vec && sg.g.outer == 1) {
        const unsigned by = (unsigned)(sg.g.nblocks < 65535 ? sg.g.nblocks : 65535);
        hipLaunchKernelGGL(block_slice_max_kernel, dim3(sg.slices, by), dim3(kThreads), 0, stream, u32(in), partial, sg);
    } else if (vec)
        hipLaunchKernelGGL((block_partial_max_kernel<true>), grid, dim3(kThreads), 0, stream, u32(in), partial, sg);
    else
        hipLaunchKernelGGL((block_partial_max_kernel<false>), grid, dim3(kThreads), 0, stream, u32(in), partial, sg);
    if (sg.slices >= 32)
        hipLaunchKernelGGL(block_fold_partials_wide_kernel, folded(nblocks), dim3(kThreads), 0, stream, partial, block_max, nblocks,
                           sg.slices);
    else if (sg.slices > 1)
        hipLaunchKernelGGL(block_fold_partials_kernel, folded((nblocks + kThreads - 1) / kThreads), dim3(kThreads), 0, stream,
                           partial, block_max, nblocks, sg.slices);
    return launch_status();
}

int qsim_block_quantize_with_max(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks,
                                 uint64_t inner, uint64_t index0, int wl, int rounding, uint32_t flags, uint64_t seed,
                                 uint32_t stream_id, const uint32_t* block_max, void* hip_stream)
{
    if (!valid_rounding(rounding)) return QSIM_ERR_ROUNDING;
    if (!valid_block_wl(wl) || !valid_flags(flags)) return QSIM_ERR_FORMAT;
    if (n > kMaxElements || !valid_index0(index0)) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!valid_block_shape(n, outer, nblocks, inner)) return QSIM_ERR_SHAPE;
    if (!in || !out || !block_max) return QSIM_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_ERR_OVERLAP;
    if (nblocks > 0x7fffffffull) return QSIM_ERR_UNSUPPORTED;
    if (ranges_overlap(block_max, nblocks * sizeof(uint32_t), in, n * 4) ||
        ranges_overlap(block_max, nblocks * sizeof(uint32_t), out, n * 4))
        return QSIM_ERR_OVERLAP;
    const SliceGeom sg = two_pass_geometry(block_schedule(n, outer, nblocks, inner));
    const RngKey key = make_key(seed, stream_id, index0);
    const int symmetric = (flags & QSIM_SYMMETRIC) ? 1 : 0;
    hipStream_t stream = as_stream(hip_stream);
    switch (rounding) {
    case QSIM_RN_EVEN: return launch_block_given_max<QSIM_RN_EVEN>(in, out, sg, wl, symmetric, key, block_max, stream);
    case QSIM_RN_AWAY: return launch_block_given_max<QSIM_RN_AWAY>(in, out, sg, wl, symmetric, key, block_max, stream);
    case QSIM_RN_ZERO: return launch_block_given_max<QSIM_RN_ZERO>(in, out, sg, wl, symmetric, key, block_max, stream);
    default:           return launch_block_given_max<QSIM_STOCHASTIC>(in, out, sg, wl, symmetric, key, block_max, stream);
    }
}

// Validation of one tensor of the SGD step.  w_q may be NULL or w_master itself.
static int check_sgd_tensor(const float* w_master, const float* w_q, const float* grad, const float* mom, uint64_t n)
{
    if (n > kMaxElements) return QSIM_ERR_SHAPE;
    if (n == 0) return QSIM_OK;
    if (!w_master || !grad || !mom) return QSIM_ERR_NULL;
    if (any_overlap(w_master, grad, n) || any_overlap(w_master, mom, n) || any_overlap(grad, mom, n))
        return QSIM_ERR_OVERLAP;
    if (w_q && (partial_overlap(w_q, w_master, n) || any_overlap(w_q, grad, n) || any_overlap(w_q, mom, n)))
        return QSIM_ERR_OVERLAP;
    return QSIM_OK;
}

static SgdHyper make_hyper(float lr, float momentum, const qsim_sgd_options* opt)
{
    SgdHyper h;
    h.lr = lr;
    h.momentum = momentum;
    h.weight_decay = opt ? opt->weight_decay : 0.0f;
    h.keep = 1.0f - (opt ? opt->dampening : 0.0f);
    h.has_decay = (opt && opt->weight_decay != 0.0f) ? 1 : 0;
    h.has_dampening = (opt && opt->dampening != 0.0f) ? 1 : 0;
    h.nesterov = (opt && opt->nesterov) ? 1 : 0;
    return h;
}

int qsim_quant_sgd_step(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n, float lr,
                        float momentum, const qsim_format* fmt_grad, const qsim_format* fmt_mom,
                        const qsim_format* fmt_weight, uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    return qsim_quant_sgd_step_ex(w_master, w_q, grad, mom, n, lr, momentum, nullptr, fmt_grad, fmt_mom, fmt_weight, seed,
                                  stream_id, hip_stream);
}

int qsim_quant_sgd_step_multi(int ntensors, float* const* w_master, float* const* w_q, const float* const* grad,
                              float* const* mom, const uint64_t* n, float lr, float momentum,
                              const qsim_format* fmt_grad, const qsim_format* fmt_mom, const qsim_format* fmt_weight,
                              uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    return qsim_quant_sgd_step_multi_ex(ntensors, w_master, w_q, grad, mom, n, lr, momentum, nullptr, fmt_grad, fmt_mom,
                                        fmt_weight, seed, stream_id, hip_stream);
}

int qsim_quant_sgd_step_ex(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n, float lr,
                           float momentum, const qsim_sgd_options* options, const qsim_format* fmt_grad,
                           const qsim_format* fmt_mom, const qsim_format* fmt_weight, uint64_t seed,
                           uint32_t stream_id, void* hip_stream)
{
    return qsim_quant_sgd_step_at(w_master, w_q, grad, mom, n, 0, lr, momentum, options, fmt_grad, fmt_mom, fmt_weight, seed,
                                  stream_id, hip_stream);
}

int qsim_quant_sgd_step_at(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n, uint64_t index0,
                           float lr, float momentum, const qsim_sgd_options* options, const qsim_format* fmt_grad,
                           const qsim_format* fmt_mom, const qsim_format* fmt_weight, uint64_t seed,
                           uint32_t stream_id, void* hip_stream)
{
    FormatPlan fg, fm, fw;
    int status;
    if ((status = make_format_plan(fmt_grad, &fg)) != QSIM_OK) return status;
    if ((status = make_format_plan(fmt_mom, &fm)) != QSIM_OK) return status;
    if ((status = make_format_plan(fmt_weight, &fw)) != QSIM_OK) return status;
    if (!valid_index0(index0)) return QSIM_ERR_SHAPE;
    for (const FormatPlan* f : {&fg, &fm, &fw})       // a shard holds whole chunks
        if (f->kind == 3 && index0 % (4ull * (uint64_t)f->lanes) != 0) return QSIM_ERR_SHAPE;
    if ((status = check_sgd_tensor(w_master, w_q, grad, mom, n)) != QSIM_OK) return status;
    if (n == 0) return QSIM_OK;
    const RngKey key = make_key(seed, stream_id, index0);
    const uint64_t groups = (n + 3) / 4;
    const uint64_t tiles = (groups + kThreads - 1) / kThreads;
    const unsigned blocks = (unsigned)(tiles < kGridX ? tiles : kGridX);       // the kernel strides over the tiles
    const bool vec = aligned16(w_master) && aligned16(grad) && aligned16(mom) && (!w_q || aligned16(w_q));
    const SgdHyper h = make_hyper(lr, momentum, options);
    hipStream_t stream = as_stream(hip_stream);
    if (vec)
        hipLaunchKernelGGL((sgd_step_kernel<true>), dim3(blocks), dim3(kThreads), 0, stream, u32(w_master), u32(w_q), u32(grad),
                           u32(mom), n, tiles, h, fg, fm, fw, key);
    else
        hipLaunchKernelGGL((sgd_step_kernel<false>), dim3(blocks), dim3(kThreads), 0, stream, u32(w_master), u32(w_q), u32(grad),
                           u32(mom), n, tiles, h, fg, fm, fw, key);
    return launch_status();
}

int qsim_quant_sgd_step_multi_ex(int ntensors, float* const* w_master, float* const* w_q, const float* const* grad,
                                 float* const* mom, const uint64_t* n, float lr, float momentum,
                                 const qsim_sgd_options* options, const qsim_format* fmt_grad,
                                 const qsim_format* fmt_mom, const qsim_format* fmt_weight, uint64_t seed,
                                 uint32_t stream_id, void* hip_stream)
{
    FormatPlan fg, fm, fw;
    int status;
    if ((status = make_format_plan(fmt_grad, &fg)) != QSIM_OK) return status;
    if ((status = make_format_plan(fmt_mom, &fm)) != QSIM_OK) return status;
    if ((status = make_format_plan(fmt_weight, &fw)) != QSIM_OK) return status;
    if (ntensors < 0) return QSIM_ERR_SHAPE;
    if (ntensors == 0) return QSIM_OK;
    if (!w_master || !grad || !mom || !n) return QSIM_ERR_NULL;
    for (int t = 0; t < ntensors; ++t) {
        status = check_sgd_tensor(w_master[t], w_q ? w_q[t] : nullptr, grad[t], mom[t], n[t]);
        if (status != QSIM_OK) return status;
    }
    const SgdHyper h = make_hyper(lr, momentum, options);
    hipStream_t stream = as_stream(hip_stream);
    // one launch per batch of up to kMultiTensors consecutive non-empty tensors (fewer than 2^31
    // tiles); entry c of a batch is tensor first + c, which is what the kernel adds to the stream
    int t = 0;
    while (t < ntensors) {
        if (n[t] == 0) {
            ++t;
            continue;
        }
        MultiTensorTable tab;
        memset(&tab, 0, sizeof(tab));
        bool vec = true;
        uint64_t tiles = 0;
        const int first = t;
        while (t < ntensors && tab.count < kMultiTensors && n[t] != 0) {
            const uint64_t groups = (n[t] + 3) / 4;
            const uint64_t mine = (groups + kThreads - 1) / kThreads;
            if (tiles + mine > kMultiTiles) break;
            const int c = tab.count++;
            tab.w_master[c] = u32(w_master[t]);
            tab.w_q[c] = w_q ? u32(w_q[t]) : nullptr;
            tab.grad[c] = u32(grad[t]);
            tab.mom[c] = u32(mom[t]);
            tab.n[c] = n[t];
            tab.first_tile[c] = (uint32_t)tiles;
            tiles += mine;
            tab.first_tile[c + 1] = (uint32_t)tiles;
            vec = vec && aligned16(w_master[t]) && aligned16(grad[t]) && aligned16(mom[t]) && (!tab.w_q[c] || aligned16(tab.w_q[c]));
            ++t;
        }
        if (tab.count == 0) {
            // a single tensor too large for a batch: the one-tensor kernel strides over its tiles
            status = qsim_quant_sgd_step_ex(w_master[t], w_q ? w_q[t] : nullptr, grad[t], mom[t], n[t], lr, momentum, options,
                                            fmt_grad, fmt_mom, fmt_weight, seed, stream_id + (uint32_t)t, hip_stream);
            if (status != QSIM_OK) return status;
            ++t;
            continue;
        }
        const RngKey key = make_key(seed, stream_id + (uint32_t)first, 0);
        if (vec) hipLaunchKernelGGL((sgd_multi_kernel<true>), folded(tiles), dim3(kThreads), 0, stream, tab, h, fg, fm, fw, key);
        else hipLaunchKernelGGL((sgd_multi_kernel<false>), folded(tiles), dim3(kThreads), 0, stream, tab, h, fg, fm, fw, key);
        if (hipGetLastError() != hipSuccess) return QSIM_ERR_LAUNCH;
    }
    return QSIM_OK;
}

// Tiles of one list, or 0 when a tensor or the total is too large.
static bool table_tiles(int ntensors, const uint64_t* n, uint64_t* tiles, int* count)
{
    *tiles = 0;
    *count = 0;
    for (int t = 0; t < ntensors; ++t) {
        if (n[t] > kMaxElements) return false;
        if (n[t] == 0) continue;
        *tiles += ((n[t] + 3) / 4 + kThreads - 1) / kThreads;
        ++*count;
    }
    return *tiles <= 0xFFFFFFFFull;
}

static size_t table_owner_offset(int count) { return ((size_t)count * sizeof(SgdTableEntry) + 15) & ~(size_t)15; }

size_t qsim_sgd_table_bytes(int ntensors, const uint64_t* n)
{
    uint64_t tiles;
    int count;
    if (ntensors <= 0 || !n || !table_tiles(ntensors, n, &tiles, &count) || count == 0) return 0;
    return table_owner_offset(count) + (((size_t)tiles * sizeof(uint32_t) + 15) & ~(size_t)15);
}

int qsim_sgd_table_build(int ntensors, float* const* w_master, float* const* w_q, const float* const* grad,
                         float* const* mom, const uint64_t* n, void* table_device, size_t table_bytes,
                         void* hip_stream, qsim_sgd_table* table)
{
    if (!table) return QSIM_ERR_NULL;
    memset(table, 0, sizeof(*table));
    if (ntensors < 0) return QSIM_ERR_SHAPE;
    if (ntensors == 0) return QSIM_OK;
    if (!w_master || !grad || !mom || !n) return QSIM_ERR_NULL;
    uint64_t tiles;
    int count;
    if (!table_tiles(ntensors, n, &tiles, &count)) return QSIM_ERR_SHAPE;
    for (int t = 0; t < ntensors; ++t) {
        const int status = check_sgd_tensor(w_master[t], w_q ? w_q[t] : nullptr, grad[t], mom[t], n[t]);
        if (status != QSIM_OK) return status;
    }
    if (count == 0) return QSIM_OK;
    const size_t need = qsim_sgd_table_bytes(ntensors, n);
    if (!table_device || !aligned16(table_device) || table_bytes < need) return QSIM_ERR_WORKSPACE;

    std::vector<unsigned char> host(need, 0);
    SgdTableEntry* entries = reinterpret_cast<SgdTableEntry*>(host.data());
    uint32_t* owner = reinterpret_cast<uint32_t*>(host.data() + table_owner_offset(count));
    bool vec = true;
    uint32_t tile = 0;
    int c = 0;
    for (int t = 0; t < ntensors; ++t) {
        if (n[t] == 0) continue;
        SgdTableEntry& e = entries[c];
        e.w_master = u32(w_master[t]);
        e.w_q = w_q ? u32(w_q[t]) : nullptr;
        e.grad = u32(grad[t]);
        e.mom = u32(mom[t]);
        e.n = n[t];
        e.first_tile = tile;
        e.position = (uint32_t)t;
        vec = vec && aligned16(w_master[t]) && aligned16(grad[t]) && aligned16(mom[t]) && (!e.w_q || aligned16(e.w_q));
        const uint32_t mine = (uint32_t)(((n[t] + 3) / 4 + kThreads - 1) / kThreads);
        for (uint32_t k = 0; k < mine; ++k) owner[tile + k] = (uint32_t)c;
        tile += mine;
        ++c;
    }
    // the host copy lives only until this function returns, so the copy is waited for
    hipStream_t stream = as_stream(hip_stream);
    if (hipMemcpyAsync(table_device, host.data(), need, hipMemcpyHostToDevice, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess) {
        (void)hipGetLastError();
        return QSIM_ERR_LAUNCH;
    }
    table->device = table_device;
    table->bytes = need;
    table->tiles = (uint32_t)tiles;
    table->count = count;
    table->aligned = vec ? 1 : 0;
    return QSIM_OK;
}

int qsim_quant_sgd_step_table(const qsim_sgd_table* table, float lr, float momentum, const qsim_sgd_options* options,
                              const qsim_format* fmt_grad, const qsim_format* fmt_mom, const qsim_format* fmt_weight,
                              uint64_t seed, uint32_t stream_id, void* hip_stream)
{
    FormatPlan fg, fm, fw;
    int status;
    if ((status = make_format_plan(fmt_grad, &fg)) != QSIM_OK) return status;
    if ((status = make_format_plan(fmt_mom, &fm)) != QSIM_OK) return status;
    if ((status = make_format_plan(fmt_weight, &fw)) != QSIM_OK) return status;
    if (!table) return QSIM_ERR_NULL;
    if (table->count == 0 || table->tiles == 0) return QSIM_OK;
    if (!table->device) return QSIM_ERR_NULL;
    if (table->count < 0 || !aligned16(table->device) ||
        table->bytes < table_owner_offset(table->count) + (size_t)table->tiles * sizeof(uint32_t))
        return QSIM_ERR_WORKSPACE;
    const SgdHyper h = make_hyper(lr, momentum, options);
    const RngKey key = make_key(seed, stream_id, 0);
    const SgdTableEntry* entries = static_cast<const SgdTableEntry*>(table->device);
    const uint32_t* owner =
        reinterpret_cast<const uint32_t*>(static_cast<const unsigned char*>(table->device) + table_owner_offset(table->count));
    hipStream_t stream = as_stream(hip_stream);
    if (table->aligned)
        hipLaunchKernelGGL((sgd_table_kernel<true>), folded(table->tiles), dim3(kThreads), 0, stream, entries, owner, table->tiles, h,
                           fg, fm, fw, key);
    else
        hipLaunchKernelGGL((sgd_table_kernel<false>), folded(table->tiles), dim3(kThreads), 0, stream, entries, owner, table->tiles, h,
                           fg, fm, fw, key);
    return launch_status();
}

void qsim_set_barrier_wait_us(uint32_t microseconds) { g_barrier_wait_us.store(microseconds, std::memory_order_relaxed); }

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
