/*
 * qsim_ref.c -- CPU ORACLE (test infrastructure only; see qsim_ref.h for the frozen rules).
 *
 * Plain scalar C in double precision.  Every step below is the definition written out: scale
 * by a power of two, floor, compare the fraction, scale back.  No shifts, no blocking, no
 * vectorisation, no code shared with the GPU library.
 */
#include "qsim_ref.h"

#include <math.h>
#include <float.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",
 * SC'11).  One round maps the counter (c0,c1,c2,c3) with round key (k0,k1) to
 *   (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0)),
 * and the key grows by the Weyl constants between rounds.
 * ---------------------------------------------------------------------------------------- */
void qsim_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint32_t qsim_ref_random_word(uint64_t seed, uint32_t stream_id, uint32_t role, uint64_t index)
{
    uint64_t j = index / 4;
    uint32_t ctr[4] = { (uint32_t)(j & 0xffffffffu), (uint32_t)(j >> 32), stream_id, role };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    qsim_ref_philox4x32_10(ctr, key, out);
    return out[index % 4];
}

/* ------------------------------------------------------------------------------------------
 * P(a, q, mode, r): the integer K with K * 2^q = a rounded to the grid 2^q (Sec. 3.1
 * "Rounding mode").  a >= 0 finite.  Returned as a double (K can exceed 2^32 when a is already
 * coarser than the grid).
 * ---------------------------------------------------------------------------------------- */
static double round_to_multiple(double a, int q, int mode, uint32_t r)
{
    double y = ldexp(a, -q);
    double k = floor(y);
    double f = y - k;
    int up = 0;
    switch (mode) {
    case QSIM_REF_RN_EVEN:    up = (f > 0.5) || (f == 0.5 && fmod(k, 2.0) != 0.0); break;
    case QSIM_REF_RN_AWAY:    up = (f >= 0.5); break;
    case QSIM_REF_RN_ZERO:    up = (f > 0.5); break;
    case QSIM_REF_STOCHASTIC: up = ((double)r < floor(ldexp(f, 32))); break;
    }
    return k + (double)up;
}

/* Attach the sign of x to the magnitude v (v >= 0, possibly above the fp32 range). */
static float with_sign_of(double v, float x)
{
    float m = (v > (double)FLT_MAX) ? INFINITY : (float)v;
    return copysignf(m, x);
}

static int valid_rounding(int rounding) { return rounding >= 0 && rounding <= 3; }
static int valid_flags(uint32_t flags)
{
    return (flags & ~(QSIM_REF_SATURATE | QSIM_REF_SUBNORMAL | QSIM_REF_SYMMETRIC)) == 0;
}
static int valid_fixed(int wl, int fl) { return wl >= 1 && wl <= 24 && fl >= wl - 128 && fl <= 149; }
static int valid_float(int e, int m) { return e >= 2 && e <= 8 && m >= 1 && m <= 23; }
static int valid_block_wl(int wl) { return wl >= 2 && wl <= 24; }

/* Do the byte ranges [a, a+n*4) and [b, b+n*4) overlap without being the same range? */
static int partial_overlap(const void* a, const void* b, uint64_t n)
{
    uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b, len = (uintptr_t)n * 4u;
    if (pa == pb) return 0;
    return (pa < pb) ? (pb - pa < len) : (pa - pb < len);
}
static int any_overlap(const void* a, const void* b, uint64_t n)
{
    return a == b || partial_overlap(a, b, n);
}

/* ------------------------------------------------------------------------------------------
 * Fixed point (wl, fl)  (Sec. 3.1 "Number Formats", second paragraph).
 * ---------------------------------------------------------------------------------------- */
static float fixed_with_grid(float x, int wl, int q, int rounding, int saturate, int symmetric,
                             uint32_t r)
{
    if (isnan(x)) return x;
    double kmax = ldexp(1.0, wl - 1) - 1.0;
    double kmin = symmetric ? -kmax : -ldexp(1.0, wl - 1);
    if (isinf(x)) {
        if (!saturate) return x;
        return (float)ldexp(x > 0 ? kmax : kmin, q);
    }
    double K = round_to_multiple(fabs((double)x), q, rounding, r);
    double Ks = signbit(x) ? -K : K;
    if (saturate) {
        if (Ks > kmax) Ks = kmax;
        if (Ks < kmin) Ks = kmin;
    }
    return with_sign_of(ldexp(fabs(Ks), q), x);
}

float qsim_ref_fixed_scalar(float x, int wl, int fl, int rounding, uint32_t flags, uint32_t r)
{
    return fixed_with_grid(x, wl, -fl, rounding, (flags & QSIM_REF_SATURATE) != 0,
                           (flags & QSIM_REF_SYMMETRIC) != 0, r);
}

/* ------------------------------------------------------------------------------------------
 * Floating point (E, M)  (Sec. 3.1 "Number Formats", first paragraph).
 * ---------------------------------------------------------------------------------------- */
float qsim_ref_float_scalar(float x, int exp_bits, int man_bits, int rounding, uint32_t flags,
                            uint32_t r)
{
    int saturate = (flags & QSIM_REF_SATURATE) != 0;
    int subnormal = (flags & QSIM_REF_SUBNORMAL) != 0;
    int bias = (1 << (exp_bits - 1)) - 1;
    int emax = bias, emin = 1 - bias;
    double maxval = ldexp(2.0 - ldexp(1.0, -man_bits), emax);

    if (isnan(x) || x == 0.0f) return x;
    if (isinf(x)) return saturate ? copysignf((float)maxval, x) : x;

    double a = fabs((double)x);
    int e = ilogb(a);
    int q = (subnormal && e < emin ? emin : e) - man_bits;
    double v = ldexp(round_to_multiple(a, q, rounding, r), q);
    if (!subnormal && v < ldexp(1.0, emin)) v = 0.0;
    if (saturate && v > maxval) v = maxval;
    return with_sign_of(v, x);
}

int qsim_ref_float_quantize_at(const float* in, float* out, uint64_t n, uint64_t index0,
                               int exp_bits, int man_bits, int rounding, uint32_t flags,
                               uint64_t seed, uint32_t stream_id)
{
    if (!valid_rounding(rounding)) return QSIM_REF_ERR_ROUNDING;
    if (!valid_float(exp_bits, man_bits) || !valid_flags(flags)) return QSIM_REF_ERR_FORMAT;
    if (n == 0) return QSIM_REF_OK;
    if (!in || !out) return QSIM_REF_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_REF_ERR_OVERLAP;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t r = 0;
        if (rounding == QSIM_REF_STOCHASTIC) r = qsim_ref_random_word(seed, stream_id, 0, index0 + i);
        out[i] = qsim_ref_float_scalar(in[i], exp_bits, man_bits, rounding, flags, r);
    }
    return QSIM_REF_OK;
}

int qsim_ref_float_quantize(const float* in, float* out, uint64_t n, int exp_bits, int man_bits,
                            int rounding, uint32_t flags, uint64_t seed, uint32_t stream_id)
{
    return qsim_ref_float_quantize_at(in, out, n, 0, exp_bits, man_bits, rounding, flags, seed,
                                      stream_id);
}

int qsim_ref_fixed_quantize_at(const float* in, float* out, uint64_t n, uint64_t index0, int wl,
                               int fl, int rounding, uint32_t flags, uint64_t seed,
                               uint32_t stream_id)
{
    if (!valid_rounding(rounding)) return QSIM_REF_ERR_ROUNDING;
    if (!valid_fixed(wl, fl) || !valid_flags(flags)) return QSIM_REF_ERR_FORMAT;
    if (n == 0) return QSIM_REF_OK;
    if (!in || !out) return QSIM_REF_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_REF_ERR_OVERLAP;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t r = 0;
        if (rounding == QSIM_REF_STOCHASTIC) r = qsim_ref_random_word(seed, stream_id, 0, index0 + i);
        out[i] = qsim_ref_fixed_scalar(in[i], wl, fl, rounding, flags, r);
    }
    return QSIM_REF_OK;
}

int qsim_ref_fixed_quantize(const float* in, float* out, uint64_t n, int wl, int fl, int rounding,
                            uint32_t flags, uint64_t seed, uint32_t stream_id)
{
    return qsim_ref_fixed_quantize_at(in, out, n, 0, wl, fl, rounding, flags, seed, stream_id);
}

/* ------------------------------------------------------------------------------------------
 * Block floating point (Sec. 3.1 "Number Formats", second paragraph).
 * ---------------------------------------------------------------------------------------- */

/* Shared exponent from the largest magnitude of a block: the fp32 exponent field of amax,
   clamped to [1, 254], minus the bias.  Non-finite amax counts as field 255 before clamping. */
static int shared_exponent(float amax)
{
    int field;
    if (isnan(amax) || isinf(amax)) field = 255;
    else if (amax < FLT_MIN) field = 0;                 /* zero or fp32 denormal */
    else field = ilogb((double)amax) + 127;
    if (field < 1) field = 1;
    if (field > 254) field = 254;
    return field - 127;
}

/* Larger of two magnitudes where NaN counts as larger than everything. */
static float max_magnitude(float acc, float x)
{
    float a = fabsf(x);
    if (isnan(acc)) return acc;
    if (isnan(a)) return a;
    return a > acc ? a : acc;
}

static int valid_block_shape(uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner)
{
    if (outer == 0 || nblocks == 0 || inner == 0) return 0;
    /* products are formed in long double range checks to stay clear of uint64 overflow */
    long double full = (long double)outer * (long double)nblocks * (long double)inner;
    if (full > 18446744073709551615.0L) return 0;
    uint64_t total = outer * nblocks * inner;
    if (outer == 1) return n <= total && n > (nblocks - 1) * inner;
    return n == total;
}

int qsim_ref_block_exponents(const float* in, uint64_t n, uint64_t outer, uint64_t nblocks,
                             uint64_t inner, int* e_s)
{
    if (n == 0) return QSIM_REF_OK;
    if (!valid_block_shape(n, outer, nblocks, inner)) return QSIM_REF_ERR_SHAPE;
    if (!in || !e_s) return QSIM_REF_ERR_NULL;
    for (uint64_t b = 0; b < nblocks; ++b) {
        float amax = 0.0f;
        for (uint64_t o = 0; o < outer; ++o)
            for (uint64_t i = 0; i < inner; ++i) {
                uint64_t idx = (o * nblocks + b) * inner + i;
                if (idx < n) amax = max_magnitude(amax, in[idx]);
            }
        e_s[b] = shared_exponent(amax);
    }
    return QSIM_REF_OK;
}

int qsim_ref_block_quantize(const float* in, float* out, uint64_t n, uint64_t outer,
                            uint64_t nblocks, uint64_t inner, int wl, int rounding, uint32_t flags,
                            uint64_t seed, uint32_t stream_id)
{
    if (!valid_rounding(rounding)) return QSIM_REF_ERR_ROUNDING;
    if (!valid_block_wl(wl) || !valid_flags(flags)) return QSIM_REF_ERR_FORMAT;
    if (n == 0) return QSIM_REF_OK;
    if (!valid_block_shape(n, outer, nblocks, inner)) return QSIM_REF_ERR_SHAPE;
    if (!in || !out) return QSIM_REF_ERR_NULL;
    if (partial_overlap(in, out, n)) return QSIM_REF_ERR_OVERLAP;
    int symmetric = (flags & QSIM_REF_SYMMETRIC) != 0;
    for (uint64_t b = 0; b < nblocks; ++b) {
        /* first the whole block's maximum (raw input), then every element of the block */
        float amax = 0.0f;
        for (uint64_t o = 0; o < outer; ++o)
            for (uint64_t i = 0; i < inner; ++i) {
                uint64_t idx = (o * nblocks + b) * inner + i;
                if (idx < n) amax = max_magnitude(amax, in[idx]);
            }
        int q = shared_exponent(amax) + 2 - wl;
        for (uint64_t o = 0; o < outer; ++o)
            for (uint64_t i = 0; i < inner; ++i) {
                uint64_t idx = (o * nblocks + b) * inner + i;
                if (idx >= n) continue;
                uint32_t r = 0;
                if (rounding == QSIM_REF_STOCHASTIC) r = qsim_ref_random_word(seed, stream_id, 0, idx);
                out[idx] = fixed_with_grid(in[idx], wl, q, rounding, 1, symmetric, r);
            }
    }
    return QSIM_REF_OK;
}

/* ------------------------------------------------------------------------------------------
 * Quantized SGD with momentum (Sec. 3.1 "Front-end interface": weight, gradient and
 * accumulator each quantized by the optimizer; Sec. 1 footnote 1: the high-precision copy).
 * ---------------------------------------------------------------------------------------- */
static int valid_format(const qsim_ref_format* f, int* status)
{
    if (!f) { *status = QSIM_REF_ERR_NULL; return 0; }
    if (!valid_rounding(f->rounding)) { *status = QSIM_REF_ERR_ROUNDING; return 0; }
    int ok = 0;
    switch (f->kind) {
    case 0: ok = 1; break;
    case 1: ok = valid_float(f->a, f->b); break;
    case 2: ok = valid_fixed(f->a, f->b); break;
    case 3: ok = valid_block_wl(f->a) && f->b >= 4 && f->b <= 1024 && (f->b & (f->b - 1)) == 0; break;
    default: ok = 0;
    }
    if (!ok || !valid_flags(f->flags)) { *status = QSIM_REF_ERR_FORMAT; return 0; }
    return 1;
}

/* Quantize a whole array in place with one format; `role` selects the random stream and the
   array index is the element index. */
static void quantize_array(float* x, uint64_t n, const qsim_ref_format* f, uint64_t seed,
                           uint32_t stream_id, uint32_t role)
{
    int stochastic = (f->rounding == QSIM_REF_STOCHASTIC);
    if (f->kind == 0) return;
    if (f->kind == 3) {
        uint64_t L = (uint64_t)f->b;
        int symmetric = (f->flags & QSIM_REF_SYMMETRIC) != 0;
        for (uint64_t c0 = 0; c0 < n; c0 += L) {
            uint64_t c1 = (c0 + L < n) ? c0 + L : n;
            float amax = 0.0f;
            for (uint64_t i = c0; i < c1; ++i) amax = max_magnitude(amax, x[i]);
            int q = shared_exponent(amax) + 2 - f->a;
            for (uint64_t i = c0; i < c1; ++i) {
                uint32_t r = stochastic ? qsim_ref_random_word(seed, stream_id, role, i) : 0;
                x[i] = fixed_with_grid(x[i], f->a, q, f->rounding, 1, symmetric, r);
            }
        }
        return;
    }
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t r = stochastic ? qsim_ref_random_word(seed, stream_id, role, i) : 0;
        x[i] = (f->kind == 1)
                   ? qsim_ref_float_scalar(x[i], f->a, f->b, f->rounding, f->flags, r)
                   : qsim_ref_fixed_scalar(x[i], f->a, f->b, f->rounding, f->flags, r);
    }
}

int qsim_ref_quant_sgd_step_ex(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n,
                               float lr, float momentum, const qsim_ref_sgd_options* opt,
                               const qsim_ref_format* fmt_grad, const qsim_ref_format* fmt_mom,
                               const qsim_ref_format* fmt_weight, uint64_t seed, uint32_t stream_id)
{
    int status = QSIM_REF_OK;
    if (!valid_format(fmt_grad, &status) || !valid_format(fmt_mom, &status) ||
        !valid_format(fmt_weight, &status))
        return status;
    if (n == 0) return QSIM_REF_OK;
    if (!w_master || !grad || !mom) return QSIM_REF_ERR_NULL;
    if (any_overlap(w_master, grad, n) || any_overlap(w_master, mom, n) || any_overlap(grad, mom, n))
        return QSIM_REF_ERR_OVERLAP;
    if (w_q && (partial_overlap(w_q, w_master, n) || any_overlap(w_q, grad, n) || any_overlap(w_q, mom, n)))
        return QSIM_REF_ERR_OVERLAP;
    const float weight_decay = opt ? opt->weight_decay : 0.0f;
    const float dampening = opt ? opt->dampening : 0.0f;
    const int nesterov = opt ? opt->nesterov : 0;

    /* gq = Qg(grad): the gradient array is an input only, so its quantized copy is a temporary */
    float* d = (float*)malloc((size_t)n * sizeof(float));
    if (!d) return QSIM_REF_ERR_ALLOC;
    memcpy(d, grad, (size_t)n * sizeof(float));
    quantize_array(d, n, fmt_grad, seed, stream_id, 0);

    /* d = gq + weight_decay * w  (on the weight the optimizer holds) */
    if (weight_decay != 0.0f)
        for (uint64_t i = 0; i < n; ++i) d[i] = fmaf(weight_decay, w_master[i], d[i]);

    /* v = Qm(momentum * v + (1 - dampening) * d) */
    if (dampening != 0.0f) {
        const float keep = 1.0f - dampening;
        for (uint64_t i = 0; i < n; ++i) mom[i] = fmaf(momentum, mom[i], keep * d[i]);
    } else {
        for (uint64_t i = 0; i < n; ++i) mom[i] = fmaf(momentum, mom[i], d[i]);
    }
    quantize_array(mom, n, fmt_mom, seed, stream_id, 1);

    /* w = w - lr * v, or with Nesterov momentum w - lr * (d + momentum * v): fp32, not quantized */
    if (nesterov)
        for (uint64_t i = 0; i < n; ++i) w_master[i] = fmaf(-lr, fmaf(momentum, mom[i], d[i]), w_master[i]);
    else
        for (uint64_t i = 0; i < n; ++i) w_master[i] = fmaf(-lr, mom[i], w_master[i]);
    free(d);

    /* w_q = Qw(w); when w_q is w_master itself the weights are kept in the weight format */
    if (w_q) {
        if (w_q != w_master) memcpy(w_q, w_master, (size_t)n * sizeof(float));
        quantize_array(w_q, n, fmt_weight, seed, stream_id, 2);
    }
    return QSIM_REF_OK;
}

int qsim_ref_quant_sgd_step(float* w_master, float* w_q, const float* grad, float* mom, uint64_t n,
                            float lr, float momentum, const qsim_ref_format* fmt_grad,
                            const qsim_ref_format* fmt_mom, const qsim_ref_format* fmt_weight,
                            uint64_t seed, uint32_t stream_id)
{
    return qsim_ref_quant_sgd_step_ex(w_master, w_q, grad, mom, n, lr, momentum, NULL, fmt_grad, fmt_mom,
                                      fmt_weight, seed, stream_id);
}
