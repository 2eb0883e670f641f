/*
 * qsim.h -- C-ABI of libqsim: fused quantize-and-round kernels for MI355X (gfx950).
 *
 * The library simulates low-precision number formats the way arXiv 1910.04540 (QPyTorch)
 * describes in Sec. 3: a low-precision number is stored as the fp32 number it equals, so
 * every call maps an fp32 array onto the values a format can represent, in one fused kernel
 * appended after a regular fp32 operation (Sec. 3.2, the "two-kernel approach").
 *
 * Conventions shared by all entry points
 *   - Every data pointer is a DEVICE pointer owned by the caller.  Format descriptors
 *     (qsim_format) are HOST pointers, read before the call returns.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued on it and the call returns without synchronising (qsim_sgd_table_build excepted),
 *     so calls can be recorded by a stream capture into a HIP graph: every call is kernel launches
 *     only.  The first qsim_block_quantize of a single-pass shape on a device asks the runtime for
 *     the kernel's occupancy once; make that first call outside a capture.
 *   - The library allocates and frees no device memory.  Scratch memory and tables, where needed,
 *     are the caller's (`workspace`, `table_device`); qsim_block_quantize_static alone uses an
 *     array of fixed size that is part of the library's image on the device.
 *   - in == out (exactly the same array) is allowed; any other overlap between arrays of one
 *     call is rejected with QSIM_ERR_OVERLAP.
 *   - n == 0 is a successful no-op.  n is limited to 2^38 elements.
 *   - Return value: a QSIM_* status; 0 = success.  Arguments are validated in the order
 *     rounding, format/flags, shape, n == 0, null pointers, overlap, workspace; nothing is
 *     launched when validation fails.  No exception or abort crosses this boundary.
 *   - Non-finite inputs (the paper does not simulate them): NaN is returned unchanged; +-Inf is
 *     treated as larger than every finite number (the largest code when the format saturates,
 *     unchanged otherwise).
 *
 * Rounding (Sec. 3.1 "Rounding mode"): every format rounds the magnitude |x| to an integer
 * multiple K of a grid step 2^q and re-attaches the sign.  With y = |x| / 2^q, k = floor(y),
 * f = y - k:  K = k + 1 if the mode rounds up, else k.
 *     QSIM_RN_EVEN     up when f > 1/2, or f == 1/2 and k is odd
 *     QSIM_RN_AWAY     up when f >= 1/2            (ties away from zero)
 *     QSIM_RN_ZERO     up when f > 1/2             (ties toward zero)
 *     QSIM_STOCHASTIC  up when r < floor(f * 2^32), r = the element's 32-bit random word
 * Random words come from Philox4x32-10 with key = (seed mod 2^32, seed div 2^32) and counter =
 * (lo32(i div 4), hi32(i div 4), stream_id, role): element i (flat row-major index in the
 * array passed to the call) takes output word i mod 4.  role is 0 except in the SGD step.
 * Results therefore do not depend on the launch shape and are reproducible from
 * (seed, stream_id) alone.
 */
#ifndef QSIM_H
#define QSIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    QSIM_OK = 0,
    QSIM_ERR_NULL = 1,        /* a required pointer is NULL */
    QSIM_ERR_FORMAT = 2,      /* format parameters or flags out of range */
    QSIM_ERR_ROUNDING = 3,    /* rounding mode not one of the four below */
    QSIM_ERR_SHAPE = 4,       /* n does not match the block layout, or n too large */
    QSIM_ERR_OVERLAP = 5,     /* arrays overlap (other than in == out) */
    QSIM_ERR_WORKSPACE = 6,   /* workspace missing, misaligned or too small */
    QSIM_ERR_UNSUPPORTED = 7,
    QSIM_ERR_LAUNCH = 8       /* the HIP runtime refused the launch (no device, bad stream) */
};

/* Sec. 3.1 "Rounding mode". */
enum { QSIM_RN_EVEN = 0, QSIM_RN_AWAY = 1, QSIM_RN_ZERO = 2, QSIM_STOCHASTIC = 3 };

enum {
    QSIM_SATURATE = 1u,        /* clamp to the format's range instead of leaving the range open */
    QSIM_SUBNORMAL = 2u,       /* float only: gradual underflow below 2^emin instead of flush to zero */
    QSIM_SYMMETRIC = 4u,       /* fixed/block: drop the most negative two's-complement code */
    QSIM_WORKSPACE_KEPT = 8u   /* qsim_block_quantize(_at) only: the caller keeps the workspace, see there */
};

/*
 * Floating point with exp_bits exponent and man_bits mantissa bits (Sec. 3.1 "Number Formats",
 * first paragraph).  2 <= exp_bits <= 8, 1 <= man_bits <= 23.  IEEE-like: bias = 2^(E-1) - 1,
 * emax = bias, emin = 1 - bias, largest value (2 - 2^-M) * 2^emax; (5,10) is binary16, (8,7)
 * is bfloat16.  Grid step of x: 2^(e - M) with e = floor(log2 |x|); with QSIM_SUBNORMAL the
 * step stops shrinking at 2^(emin - M), without it results below 2^emin become (signed) zero.
 * QSIM_SATURATE clamps magnitudes above the largest value to it; otherwise the exponent is
 * unbounded above within the fp32 carrier.
 */
int qsim_float_quantize(const float* in, float* out, uint64_t n, int exp_bits, int man_bits,
                        int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id,
                        void* hip_stream);

/*
 * Fixed point with word length wl and fl fractional bits (Sec. 3.1 "Number Formats", second
 * paragraph).  1 <= wl <= 24, wl - 128 <= fl <= 149.  Grid step 2^-fl.  With QSIM_SATURATE the
 * integer code is clamped to [-2^(wl-1), 2^(wl-1) - 1] ([-(2^(wl-1) - 1), 2^(wl-1) - 1] with
 * QSIM_SYMMETRIC); without it the value is only rounded to the grid.
 */
int qsim_fixed_quantize(const float* in, float* out, uint64_t n, int wl, int fl, int rounding,
                        uint32_t flags, uint64_t seed, uint32_t stream_id, void* hip_stream);

/*
 * Block floating point with word length wl (Sec. 3.1 "Number Formats", second paragraph: the
 * exponent is shared across a block; a block is one index of a tensor dimension or the whole
 * tensor).  2 <= wl <= 24.  The array is viewed row-major as [outer, nblocks, inner]; block b
 * is the set of elements (o, b, i).  Whole tensor: (1, 1, n).  Leading dimension of [R, C]:
 * (1, R, C).  Contiguous chunks of L: (1, ceil(n / L), L), where the last chunk may be short.
 * n must equal outer * nblocks * inner unless outer == 1.
 * Per block: e_s = the fp32 exponent field of the largest |x| in the block, clamped to
 * [1, 254], minus 127; grid step 2^(e_s + 2 - wl); integer codes always clamped to
 * [-2^(wl-1), 2^(wl-1) - 1] (QSIM_SYMMETRIC as above).  The maximum is taken on the raw input.
 *
 * workspace: device scratch of at least qsim_block_workspace_bytes(...) bytes, 16-byte
 * aligned, used when a block is spread over several workgroups; may be NULL when that function
 * returns 0.  Its contents are overwritten; it needs no initialisation, and no two calls that are
 * in flight at the same time may share it.
 *
 * QSIM_WORKSPACE_KEPT (in `flags`).  The single-pass forms (see qsim_set_barrier_wait_us) keep a
 * few counters in the workspace that must be zero when their kernel starts.  By default every such
 * call zeroes them with a small launch of its own before the kernel.  A caller that sets a
 * workspace aside for the calls of ONE shape (n, outer, nblocks, inner) saves that launch: fill the
 * workspace with zeros once, before its first use, and pass QSIM_WORKSPACE_KEPT with every call
 * that uses it.  Each call then leaves the workspace ready for the next one (also when it is
 * replayed from a graph, and also when its bounded wait ran out), provided that nothing but
 * qsim_block_quantize(_at) calls of that shape, all with this flag, writes to it in between.
 * The flag changes no result.  Forms that need no such state ignore it.
 * The first 32-bit word of the workspace counts, since the workspace was last zeroed, the
 * workgroups of single-pass calls that stopped waiting for the others (qsim_set_barrier_wait_us);
 * it is there for callers and tests that want to know that this happened.
 */
int qsim_block_quantize(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks,
                        uint64_t inner, int wl, int rounding, uint32_t flags, uint64_t seed,
                        uint32_t stream_id, void* workspace, size_t workspace_bytes,
                        void* hip_stream);
size_t qsim_block_workspace_bytes(uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner);

/*
 * qsim_block_quantize for callers that cannot provide device memory of their own for the scratch and
 * cannot allocate it either: code under a stream capture, tight serving loops, harnesses that
 * forbid allocation.  Same arguments and results as qsim_block_quantize without the workspace:
 * the scratch is an array of QSIM_STATIC_SCRATCH_BYTES that the library holds in device memory on
 * every GPU it runs on, from the time it is loaded until the process ends.  The call allocates and
 * frees nothing and launches kernels only (it clears what it needs of the array with a kernel of
 * its own first, so what an earlier call left there does not matter).
 *   - A shape whose qsim_block_workspace_bytes exceeds QSIM_STATIC_SCRATCH_BYTES is rejected with
 *     QSIM_ERR_WORKSPACE; nothing is launched.
 *   - QSIM_WORKSPACE_KEPT is not accepted here (QSIM_ERR_FORMAT).
 *   - All calls on one GPU share the one array: two such calls that are in flight on that GPU at
 *     the same time (two streams, two threads) race and give undefined results.  Calls on one
 *     stream, or otherwise ordered one after the other, are fine.
 *   - The first call on a device looks the array's address up (and, for a single-pass shape, asks
 *     for the kernel's occupancy); neither allocates.
 */
#define QSIM_STATIC_SCRATCH_BYTES (4u << 20)
int qsim_block_quantize_static(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks,
                               uint64_t inner, int wl, int rounding, uint32_t flags, uint64_t seed,
                               uint32_t stream_id, void* hip_stream);

/*
 * Tuning and test knob of qsim_block_quantize.  A block that is too long for one workgroup but
 * fits in the register files of the chip (a whole tensor of up to 16 Mi elements; in larger
 * tensors every block of up to 8 Mi elements, contiguous or strided) is quantized in a single
 * pass by workgroups that hold its slices in registers and wait for each other once.  For a whole
 * tensor the grid is no larger than what the device holds at once; for many blocks the workgroups
 * are numbered block by block and the forms count on the device starting them in that order, so
 * that the workgroups of the lowest unfinished block are always running.  Neither holds when the
 * device is shared with other work (other processes, other streams), so the wait is bounded: after
 * `microseconds` (default 2000) a workgroup stops waiting and derives the missing maxima from
 * memory itself.  The result is the same, only slower: a call that normally takes tens of
 * microseconds then takes `microseconds` and more.  Such workgroups are counted in the first word of
 * the workspace (see qsim_block_quantize).  0 makes every workgroup take that path at once.
 * Process-wide: it affects every call made after it returns, on any thread.
 */
void qsim_set_barrier_wait_us(uint32_t microseconds);

/* A number format for one category of numbers in the optimizer (Sec. 3.1 "Front-end interface"). */
typedef struct {
    int kind;       /* 0 identity (fp32), 1 float, 2 fixed, 3 block over contiguous chunks */
    int a;          /* exp_bits | wl | wl */
    int b;          /* man_bits | fl | chunk length L: a power of two, 4 <= L <= 1024 */
    int rounding;   /* QSIM_RN_* or QSIM_STOCHASTIC */
    uint32_t flags; /* QSIM_SATURATE | QSIM_SUBNORMAL | QSIM_SYMMETRIC */
} qsim_format;

/*
 * Fused low-precision SGD-with-momentum step (Sec. 3.1 "Front-end interface": weight, gradient
 * and accumulator are quantized by the optimizer, each with its own format; Sec. 1 footnote 1:
 * an fp32 master copy of the weights accumulates the updates).  One pass, per element i:
 *     gq        = Qg(grad[i])
 *     v         = Qm(fma(momentum, mom[i], gq));     mom[i] = v
 *     w         = fma(-lr, v, w_master[i]);          w_master[i] = w      (not quantized)
 *     w_q[i]    = Qw(w)                              (skipped when w_q is NULL)
 * Both fma are single-rounding fp32 operations.  A block-kind format groups the array it
 * quantizes into contiguous chunks of L elements (the last may be short).  Random words use
 * role 0 for the gradient, 1 for the momentum and 2 for the weight.  Weight decay, dampening and
 * Nesterov momentum are in qsim_quant_sgd_step_ex.  w_master and mom are updated in place; grad is read only.
 * w_q may also be w_master itself: then no fp32 master copy is kept and the weights are stored in
 * the weight format (the accumulator is quantized, as the paper's optimizer does by default).
 */
int qsim_quant_sgd_step(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n,
                        float lr, float momentum, const qsim_format* fmt_grad,
                        const qsim_format* fmt_mom, const qsim_format* fmt_weight, uint64_t seed,
                        uint32_t stream_id, void* hip_stream);

/*
 * The same step over `ntensors` tensors in one launch per 64 tensors (a model's parameters are many,
 * mostly small tensors; one launch each would be bound by launch latency).  w_master, w_q, grad,
 * mom and n are HOST arrays of `ntensors` device pointers / element counts; w_q may be NULL (no
 * quantized copies) and so may any of its entries.  Tensor t is processed exactly as
 * qsim_quant_sgd_step would with stream_id + t, so results do not depend on how tensors are grouped.
 * Overlap is checked within each tensor, not between tensors.  Empty tensors are skipped.
 * This form needs no set-up, and each of its launches pays its own start and drain; for a list
 * that stays the same from step to step (an optimizer's) qsim_quant_sgd_step_table below is the
 * fast form: one launch, whatever the length of the list (161 tensors of a ResNet-50: 99 us
 * against 122 us).
 */
int qsim_quant_sgd_step_multi(int ntensors, float* const* w_master, float* const* w_q,
                              const float* const* grad, float* const* mom, const uint64_t* n, float lr,
                              float momentum, const qsim_format* fmt_grad, const qsim_format* fmt_mom,
                              const qsim_format* fmt_weight, uint64_t seed, uint32_t stream_id,
                              void* hip_stream);

/*
 * The optional terms of PyTorch-style SGD in the fused step (NULL or all zero = the plain step).
 * Each is one fp32 operation per element, placed between the quantizers as follows:
 *     gq = Qg(grad[i])
 *     d  = fma(weight_decay, w_master[i], gq)                    skipped when weight_decay == 0
 *     v  = Qm(fma(momentum, mom[i], (1 - dampening) * d))        the product skipped when dampening == 0
 *     w  = fma(-lr, nesterov ? fma(momentum, v, d) : v, w_master[i])
 *     w_q[i] = Qw(w)
 * 1 - dampening is formed in fp32.  Weight decay acts on the weight the optimizer holds (w_master).
 */
typedef struct {
    float weight_decay;
    float dampening;
    int nesterov;       /* 0 or 1 */
} qsim_sgd_options;

int qsim_quant_sgd_step_ex(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n, float lr,
                           float momentum, const qsim_sgd_options* options, const qsim_format* fmt_grad,
                           const qsim_format* fmt_mom, const qsim_format* fmt_weight, uint64_t seed,
                           uint32_t stream_id, void* hip_stream);
int qsim_quant_sgd_step_multi_ex(int ntensors, float* const* w_master, float* const* w_q,
                                 const float* const* grad, float* const* mom, const uint64_t* n, float lr,
                                 float momentum, const qsim_sgd_options* options,
                                 const qsim_format* fmt_grad, const qsim_format* fmt_mom,
                                 const qsim_format* fmt_weight, uint64_t seed, uint32_t stream_id,
                                 void* hip_stream);

/*
 * Shards.  When the arrays of a call hold elements index0 .. index0 + n - 1 of a larger tensor (one
 * GPU's share of it), the `_at` forms key the random words by the element's index in the WHOLE
 * tensor, so the shards of a tensor, quantized separately in any split, give exactly what one call
 * on the whole tensor gives.  index0 must be a multiple of 4 and at most 2^62 (QSIM_ERR_SHAPE
 * otherwise); everything else is as in the plain form, which is the `_at` form with index0 == 0.
 *
 *   qsim_float_quantize_at, qsim_fixed_quantize_at   any split at multiples of 4.
 *   qsim_block_quantize_at   the shard holds WHOLE blocks (rows of a per-row format); the shape
 *                            arguments describe the shard.
 *   qsim_quant_sgd_step_at   a shard of the parameters; index0 must also be a multiple of the chunk
 *                            length of every block format, so that the shard holds whole chunks.
 *
 * Blocks that are split over shards (the whole tensor as one block, blocks along a dimension that is
 * sharded) need the block maxima of all shards before anything can be rounded:
 *
 *   qsim_block_max   block_max[b] = the largest |x| of block b within THIS array, as the bit pattern
 *                    of that fp32 magnitude (so the maximum over shards is the elementwise maximum
 *                    of these unsigned integers: a max-all-reduce of nblocks words); 0 for an empty
 *                    range.  block_max: nblocks words of device memory.  workspace as for
 *                    qsim_block_quantize with the same shape.  n == 0 is QSIM_ERR_SHAPE here.
 *   qsim_block_quantize_with_max   the second half: quantizes with the given block maxima (device
 *                    memory, nblocks words, read only) instead of the array's own.
 *
 * With block_max from qsim_block_max on the same array and index0 == 0 the pair gives exactly what
 * qsim_block_quantize gives.
 */
int qsim_float_quantize_at(const float* in, float* out, uint64_t n, uint64_t index0, int exp_bits,
                           int man_bits, int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id,
                           void* hip_stream);
int qsim_fixed_quantize_at(const float* in, float* out, uint64_t n, uint64_t index0, int wl, int fl,
                           int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id,
                           void* hip_stream);
int qsim_block_quantize_at(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks,
                           uint64_t inner, uint64_t index0, int wl, int rounding, uint32_t flags,
                           uint64_t seed, uint32_t stream_id, void* workspace, size_t workspace_bytes,
                           void* hip_stream);
int qsim_quant_sgd_step_at(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n,
                           uint64_t index0, float lr, float momentum, const qsim_sgd_options* options,
                           const qsim_format* fmt_grad, const qsim_format* fmt_mom,
                           const qsim_format* fmt_weight, uint64_t seed, uint32_t stream_id,
                           void* hip_stream);
int qsim_block_max(const float* in, uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner,
                   uint32_t* block_max, void* workspace, size_t workspace_bytes, void* hip_stream);
int qsim_block_quantize_with_max(const float* in, float* out, uint64_t n, uint64_t outer, uint64_t nblocks,
                                 uint64_t inner, uint64_t index0, int wl, int rounding, uint32_t flags,
                                 uint64_t seed, uint32_t stream_id, const uint32_t* block_max,
                                 void* hip_stream);

/*
 * The same step over a FIXED list of tensors of any length in ONE launch (an optimizer steps the
 * same parameter, gradient and momentum tensors every iteration): the list is written once into a
 * table in device memory, and every later step only names the table.
 *
 *   qsim_sgd_table_bytes   size of the table for these element counts (0 for an empty list, and
 *                          for a list qsim_sgd_table_build would reject with QSIM_ERR_SHAPE).
 *   qsim_sgd_table_build   validates the list exactly as qsim_quant_sgd_step_multi does, writes the
 *                          table into `table_device` (DEVICE memory of the caller, 16-byte aligned,
 *                          at least qsim_sgd_table_bytes; else QSIM_ERR_WORKSPACE) with a copy on
 *                          `hip_stream`, WAITS for that copy, and fills the host descriptor *table.
 *                          More than 2^32 - 1 tiles of 1024 elements in total: QSIM_ERR_SHAPE.
 *   qsim_quant_sgd_step_table   tensor t of the list is processed exactly as qsim_quant_sgd_step_ex
 *                          would with stream_id + t (t counts empty tensors too), so the result is
 *                          that of qsim_quant_sgd_step_multi_ex on the same list.
 *
 * The caller keeps the table's memory and the tensors alive and unchanged in place while the
 * descriptor is in use; a descriptor not filled by qsim_sgd_table_build is QSIM_ERR_NULL /
 * QSIM_ERR_WORKSPACE at best and undefined otherwise.  An empty list (or only empty tensors) builds
 * a descriptor whose step is a no-op.
 */
typedef struct {
    const void* device;     /* the table (device memory of the caller) */
    size_t bytes;           /* its size */
    uint32_t tiles;         /* workgroups of one step */
    int32_t count;          /* non-empty tensors */
    int32_t aligned;        /* 1 when every array is 16-byte aligned */
} qsim_sgd_table;

size_t qsim_sgd_table_bytes(int ntensors, const uint64_t* n);
int qsim_sgd_table_build(int ntensors, float* const* w_master, float* const* w_q, const float* const* grad,
                         float* const* mom, const uint64_t* n, void* table_device, size_t table_bytes,
                         void* hip_stream, qsim_sgd_table* table);
int qsim_quant_sgd_step_table(const qsim_sgd_table* table, float lr, float momentum,
                              const qsim_sgd_options* options, const qsim_format* fmt_grad,
                              const qsim_format* fmt_mom, const qsim_format* fmt_weight, uint64_t seed,
                              uint32_t stream_id, void* hip_stream);

/* Static description of a status code (never NULL). */
const char* qsim_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif
