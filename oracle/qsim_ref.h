/*
 * qsim_ref.h -- CPU ORACLE for the low-precision quantizers.  TEST INFRASTRUCTURE ONLY.
 *
 * This is the slow, plain definition of what the GPU library must compute.  It is used by the
 * tests, by the smoke check and as the reported CPU baseline of the benchmark; nothing in the
 * product path may call it.  It shares no code with the GPU library.  All pointers are HOST
 * pointers.  Arithmetic is done in double precision with ldexp/floor, never with shifts.
 *
 * The paper (arXiv 1910.04540, Sec. 3.1 "Number Formats" and "Rounding mode") names the formats and
 * rounding modes in prose only: it prints no formula and no worked example.  The numerical rules
 * below are therefore the frozen reading of those passages; every choice the paper leaves open
 * is listed here.
 *
 * Carrier (Sec. 3, first paragraph): a low-precision number is stored as the fp32 number it
 * equals.  Input and output are fp32 arrays; the output is always exactly representable in
 * the target format.
 *
 * ---- Rounding primitive  P(a, q, mode, r) ------------------------------------------------
 * a >= 0 finite, q integer, r one 32-bit random word.  Rounds a to an integer multiple K of 2^q:
 *     y = a * 2^-q,  k = floor(y),  f = y - k  (all exact)
 *     up = (f > 1/2) or (f == 1/2 and k odd)      QSIM_RN_EVEN   (ties to even multiple)
 *          (f >= 1/2)                              QSIM_RN_AWAY   (ties away from zero)
 *          (f > 1/2)                               QSIM_RN_ZERO   (ties toward zero)
 *          (r < floor(f * 2^32))                   QSIM_STOCHASTIC
 *     K = k + up
 * Rounding acts on the magnitude; the sign is re-attached afterwards, so "away"/"toward zero"
 * have their natural meaning and Q(-x) = -Q(x) for the same r (Sec. 3.1 "Rounding mode" lists
 * the three tie rules and stochastic rounding; it gives no default and no formula).
 * Stochastic rounding rounds up with probability floor(f*2^32)/2^32, which equals f exactly
 * whenever f has at most 32 fractional bits, so E[Q(x)] = x.  A value already on the grid has
 * f = 0 and never moves, in any mode.  Zero keeps its sign.
 *
 * ---- Fixed point (wl, fl)   (Sec. 3.1 "Number Formats", second paragraph) ----------------
 * wl = word length in bits (1..24: the carrier's 24-bit significand is the paper's stated
 * limit), fl = fractional bits (wl-128 <= fl <= 149, so that every code is a finite fp32).
 *     q = -fl;  K = P(|x|, q);  Ks = sign(x) * K
 *     QSIM_SATURATE:  Ks = clamp(Ks, Kmin, Kmax),  Kmax = 2^(wl-1) - 1,
 *                     Kmin = -2^(wl-1)  (two's complement), or -Kmax with QSIM_SYMMETRIC
 *     out = Ks * 2^-fl
 * Without QSIM_SATURATE there is no range limit (rounding to the grid only; no wrap-around).
 *
 * ---- Floating point (E, M)  (Sec. 3.1 "Number Formats", first paragraph) ------------------
 * E exponent bits (2..8), M mantissa bits (1..23), IEEE-like layout: bias = 2^(E-1) - 1,
 * emax = bias, emin = 1 - bias (the all-ones exponent code is reserved, so that (5,10) is
 * binary16 and (8,7) is bfloat16, both named by the paper), maxval = (2 - 2^-M) * 2^emax.
 * The paper's bound (exponent below 8 bits, mantissa below 23) is read inclusively because it
 * lists bfloat16 (E = 8) as supported.
 *     e = floor(log2 |x|)                      (true exponent, also for fp32 denormals)
 *     QSIM_SUBNORMAL set:   q = max(e, emin) - M      (gradual underflow)
 *     QSIM_SUBNORMAL clear: q = e - M; after rounding, a magnitude < 2^emin becomes zero
 *                           (the paper's default: it leaves denormals out)
 *     v = P(|x|, q) * 2^q                      (a carry into the next binade is automatic)
 *     QSIM_SATURATE set:   v > maxval  ->  v = maxval
 *     QSIM_SATURATE clear: the exponent is unbounded above (the paper has no Inf); only a
 *                          value above the carrier's largest finite number becomes +-Inf
 *     out = sign(x) * v
 *
 * ---- Block floating point (wl)  (Sec. 3.1 "Number Formats", second paragraph) -------------
 * The tensor is viewed row-major as [outer, nblocks, inner]; block b holds every element
 * (o, b, i).  Whole tensor as one block: outer = 1, nblocks = 1.  One block per index of the
 * leading dimension of [R, C]: outer = 1, nblocks = R, inner = C.  Contiguous chunks of L:
 * outer = 1, inner = L, nblocks = ceil(n / L) (the last chunk may be short when outer == 1).
 *     amax  = max over the block of |x_i|, taken on the raw input
 *     field = the 8-bit fp32 exponent field of amax, clamped to [1, 254]
 *     e_s   = field - 127          (shared exponent; fp32 denormals and zero use -126)
 *     q     = e_s + 2 - wl         (sign bit + one integer bit at 2^e_s + wl-2 fraction bits)
 *     K = P(|x_i|, q);  Ks = sign * K clamped to [-2^(wl-1), 2^(wl-1) - 1]  (always; or to
 *         [-Kmax, Kmax] with QSIM_SYMMETRIC);  out_i = Ks * 2^q
 * This is fixed point (wl, fl = wl - 2 - e_s) with saturation, applied per block.  wl in 2..24.
 * An all-zero block is returned unchanged (a consequence of the rule, not a special case).
 *
 * ---- Non-finite inputs (the paper does not simulate NaN and Inf) --------------------------
 * NaN: returned unchanged (same bits) by every quantizer.  +-Inf: a magnitude above every finite
 * one: +-max code when the format saturates, unchanged otherwise.  In a block, a non-finite
 * element makes field = 254 after clamping.
 *
 * ---- Random words: Philox4x32-10  (Salmon et al., SC'11) ----------------------------------
 * key = (seed mod 2^32, seed div 2^32); counter = (lo32(j), hi32(j), stream_id, role) with
 * j = i div 4, where i is the flat row-major index of the element in the tensor passed to the
 * call; element i uses output word (i mod 4).  role = 0 in the three quantizers; in the SGD step
 * 0 = gradient, 1 = momentum, 2 = weight.  One word per element, whatever the format.
 *
 * ---- Quantized SGD with momentum  (Sec. 3.1 "Front-end interface"; Sec. 1 footnote 1) ------
 * Per element, in fp32, each line rounding once:
 *     gq = Qg(grad[i])
 *     v  = Qm(fma(momentum, mom[i], gq));        mom[i] = v
 *     w  = fma(-lr, v, w_master[i]);             w_master[i] = w   (fp32 master copy)
 *     w_q[i] = Qw(w)                             (skipped when w_q is NULL; w_q may be w_master
 *                                                itself: then the weights are kept quantized)
 * A block-kind format uses contiguous chunks of L elements of the array it quantizes (for Qm the
 * array of fma results, for Qw the updated w).  The step follows the convention of PyTorch's SGD;
 * its three optional terms (qsim_ref_sgd_options) are, each one fp32 operation per line:
 *     d  = fma(weight_decay, w_master[i], gq)                 (weight decay, before the momentum)
 *     v  = Qm(fma(momentum, mom[i], (1 - dampening) * d))     (dampening; 1 - dampening in fp32)
 *     w  = fma(-lr, fma(momentum, v, d), w_master[i])         (Nesterov momentum)
 * A term whose option is zero is skipped altogether (no multiplication by one, no addition of zero).
 *
 * Return value of every function: a QSIM_* status, 0 = success.  The validation rules are those
 * of the GPU library's header.
 */
#ifndef QSIM_REF_H
#define QSIM_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    QSIM_REF_OK = 0, QSIM_REF_ERR_NULL = 1, QSIM_REF_ERR_FORMAT = 2, QSIM_REF_ERR_ROUNDING = 3,
    QSIM_REF_ERR_SHAPE = 4, QSIM_REF_ERR_OVERLAP = 5, QSIM_REF_ERR_ALLOC = 9
};
enum { QSIM_REF_RN_EVEN = 0, QSIM_REF_RN_AWAY = 1, QSIM_REF_RN_ZERO = 2, QSIM_REF_STOCHASTIC = 3 };
enum { QSIM_REF_SATURATE = 1u, QSIM_REF_SUBNORMAL = 2u, QSIM_REF_SYMMETRIC = 4u };

typedef struct {
    int kind;      /* 0 identity, 1 float, 2 fixed, 3 block over contiguous chunks */
    int a;         /* exp_bits | wl | wl */
    int b;         /* man_bits | fl | chunk length L */
    int rounding;
    uint32_t flags;
} qsim_ref_format;

/* Philox4x32-10: four output words for one counter and key. */
void qsim_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The random word of element `index` (see the header comment). */
uint32_t qsim_ref_random_word(uint64_t seed, uint32_t stream_id, uint32_t role, uint64_t index);

/* Scalar quantizers: one value, one random word. */
float qsim_ref_fixed_scalar(float x, int wl, int fl, int rounding, uint32_t flags, uint32_t r);
float qsim_ref_float_scalar(float x, int exp_bits, int man_bits, int rounding, uint32_t flags,
                            uint32_t r);

/* Array quantizers.  The `_at` forms treat in[0] as element `index0` of a larger tensor (they
   exist so that a caller may split an array over threads); the plain forms use index0 = 0. */
int qsim_ref_float_quantize_at(const float* in, float* out, uint64_t n, uint64_t index0,
                               int exp_bits, int man_bits, int rounding, uint32_t flags,
                               uint64_t seed, uint32_t stream_id);
int qsim_ref_float_quantize(const float* in, float* out, uint64_t n, int exp_bits, int man_bits,
                            int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id);
int qsim_ref_fixed_quantize_at(const float* in, float* out, uint64_t n, uint64_t index0, int wl,
                               int fl, int rounding, uint32_t flags, uint64_t seed,
                               uint32_t stream_id);
int qsim_ref_fixed_quantize(const float* in, float* out, uint64_t n, int wl, int fl, int rounding,
                            uint32_t flags, uint64_t seed, uint32_t stream_id);
int qsim_ref_block_quantize(const float* in, float* out, uint64_t n, uint64_t outer,
                            uint64_t nblocks, uint64_t inner, int wl, int rounding, uint32_t flags,
                            uint64_t seed, uint32_t stream_id);
/* Shared exponent e_s of every block, for inspection by tests (e_s[nblocks]). */
int qsim_ref_block_exponents(const float* in, uint64_t n, uint64_t outer, uint64_t nblocks,
                             uint64_t inner, int* e_s);

/* Options of the step; NULL means all zero (plain SGD with momentum). */
typedef struct {
    float weight_decay;   /* d = gq + weight_decay * w                              */
    float dampening;      /* v = Qm(momentum * v + (1 - dampening) * d)             */
    int nesterov;         /* w -= lr * (d + momentum * v)  instead of  w -= lr * v  */
} qsim_ref_sgd_options;

int qsim_ref_quant_sgd_step_ex(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n,
                               float lr, float momentum, const qsim_ref_sgd_options* opt,
                               const qsim_ref_format* fmt_grad, const qsim_ref_format* fmt_mom,
                               const qsim_ref_format* fmt_weight, uint64_t seed, uint32_t stream_id);
int qsim_ref_quant_sgd_step(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n,
                            float lr, float momentum, const qsim_ref_format* fmt_grad,
                            const qsim_ref_format* fmt_mom, const qsim_ref_format* fmt_weight,
                            uint64_t seed, uint32_t stream_id);

#ifdef __cplusplus
}
#endif
#endif
