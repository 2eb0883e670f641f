// Device-side building blocks: Philox4x32-10, branch-free rounding of fp32 values to a
// power-of-two grid, the three format rules, and wavefront reductions.  gfx950 only.
//
// Everything per element is straight-line code: the kernels are co-limited by HBM bandwidth and
// VALU issue (Philox alone is about 14 instructions per element), so every quantizer is written
// to a budget of 10-20 full-rate instructions and no divergent branch on the common path.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qsim.h"

namespace qsim {

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  The key and the two upper counter words are wave-uniform,
// so the key schedule lives in scalar registers; each 32x32->64 product is one v_mad_u64_u32.
// ---------------------------------------------------------------------------------------------
struct Words4 { uint32_t w[4]; };

__device__ __forceinline__ Words4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Words4{{c0, c1, c2, c3}};
}

// group0: group number, in the whole tensor, of the first group of the array a call is given
// (0 unless the array is a shard of a larger tensor); wave-uniform.
struct RngKey {
    uint32_t seed_lo, seed_hi, stream_id;
    uint64_t group0;
};

// Random words of the four elements 4*j .. 4*j+3 of the array (Sec. 3.1 "Rounding mode":
// stochastic rounding), which are elements 4*(group0+j) .. of the tensor the counter is keyed by.
__device__ __forceinline__ Words4 random_words(uint64_t j, const RngKey& key, uint32_t role)
{
    const uint64_t c = j + key.group0;
    return philox4x32_10((uint32_t)c, (uint32_t)(c >> 32), key.stream_id, role, key.seed_lo, key.seed_hi);
}

// Random words of the four elements i0 .. i0+3 for ANY i0: they straddle two counter values unless
// i0 is a multiple of four, so a run that is not group-aligned pays for two Philox blocks.
__device__ __forceinline__ Words4 random_words_at(uint64_t i0, const RngKey& key, uint32_t role)
{
    const uint32_t s = (uint32_t)i0 & 3u;
    const Words4 a = random_words(i0 >> 2, key, role);
    if (s == 0u) return a;
    const Words4 b = random_words((i0 >> 2) + 1u, key, role);
    Words4 r;
    r.w[0] = s == 1u ? a.w[1] : (s == 2u ? a.w[2] : a.w[3]);
    r.w[1] = s == 1u ? a.w[2] : (s == 2u ? a.w[3] : b.w[0]);
    r.w[2] = s == 1u ? a.w[3] : (s == 2u ? b.w[0] : b.w[1]);
    r.w[3] = s == 1u ? b.w[0] : (s == 2u ? b.w[1] : b.w[2]);
    return r;
}

// The same when the lanes of a wavefront hold CONSECUTIVE runs (lane l + 1 starts four elements
// after lane l, so i0 & 3 is the same in all of them): the second Philox block of a lane's run is the
// first block of the next lane's, and is taken from there instead of being drawn again.  The last
// lane has no such neighbour, so its result is only right for a group-aligned run: the caller gives
// it no elements.  Every lane of the wavefront must make the call.
__device__ __forceinline__ Words4 random_words_at_shared(uint64_t i0, const RngKey& key, uint32_t role)
{
    const uint32_t s = (uint32_t)i0 & 3u;                  // wave-uniform
    const Words4 a = random_words(i0 >> 2, key, role);
    if (s == 0u) return a;
    Words4 b;
#pragma unroll
    for (int i = 0; i < 3; ++i) b.w[i] = (uint32_t)__shfl_down((int)a.w[i], 1);
    Words4 r;
    r.w[0] = s == 1u ? a.w[1] : (s == 2u ? a.w[2] : a.w[3]);
    r.w[1] = s == 1u ? a.w[2] : (s == 2u ? a.w[3] : b.w[0]);
    r.w[2] = s == 1u ? a.w[3] : (s == 2u ? b.w[0] : b.w[1]);
    r.w[3] = s == 1u ? b.w[0] : (s == 2u ? b.w[1] : b.w[2]);
    return r;
}

// ---------------------------------------------------------------------------------------------
// Rounding a non-negative scaled value y = |x| / 2^q (y < 2^24, exact in fp32) to an integer
// (Sec. 3.1 "Rounding mode").  fract/trunc/convert are exact on such y; the stochastic threshold
// floor(f * 2^32) is exact because f has at most 24 significant bits.
// ---------------------------------------------------------------------------------------------
template <int MODE>
__device__ __forceinline__ float round_scaled(float y, uint32_t r)
{
    if (MODE == QSIM_RN_EVEN) return __builtin_rintf(y);            // v_rndne_f32
    const float f = __builtin_amdgcn_fractf(y);
    const uint32_t k = (uint32_t)y;                                 // truncation
    bool up;
    if (MODE == QSIM_RN_AWAY) up = f >= 0.5f;
    else if (MODE == QSIM_RN_ZERO) up = f > 0.5f;
    else up = r < (uint32_t)__builtin_ldexpf(f, 32);
    return (float)(k + (up ? 1u : 0u));
}

// ---------------------------------------------------------------------------------------------
// Fixed-grid quantizer: fixed point, and block floating point once the shared exponent is known
// (Sec. 3.1 "Number Formats", second paragraph).
//
// Both clamp limits are grid points, rounding is monotone and leaves grid points alone, so clamping
// the INPUT to [lo, hi] gives the same result as clamping the rounded code.  After the clamp
// y = |x| / 2^q is at most 2^23.  A format that does not saturate has lo = -Inf, hi = +Inf and
// thr = 2^(q+24): inputs of that size and above are already on the grid and are returned as they
// are (Inf included).  A saturating format has thr = +Inf, which only an infinite clamped
// magnitude fails to stay below: -Inf in a block whose most negative code is -Inf.  NaN is always
// returned as it is.  A y that underflows fp32 is below 2^-126: it rounds to zero in every mode.
// One code path serves every flag combination; the flags live in the plan's constants.
// ---------------------------------------------------------------------------------------------
struct GridPlan {
    int q;                // grid step 2^q
    float lo, hi;         // most negative and largest value (grid points), or -Inf / +Inf
    float thr;            // magnitudes not below thr are returned unchanged
    float anchor;         // 2^(q+23) when every input is known to be finite and that power exists, else 0
    int finite;           // every input is known to be finite: nothing is returned unchanged
};

constexpr int kClassNaN = 0x003;

template <int MODE>
__device__ __forceinline__ uint32_t quantize_to_grid(uint32_t bits, const GridPlan& p, uint32_t r)
{
    const float x = __uint_as_float(bits);
    const float a = __builtin_fabsf(__builtin_amdgcn_fmed3f(x, p.lo, p.hi));
    const float y = __builtin_ldexpf(a, -p.q);
    const float v = __builtin_ldexpf(round_scaled<MODE>(y, r), p.q);
    const uint32_t res = (__float_as_uint(v) & 0x7fffffffu) | (bits & 0x80000000u);
    const bool keep = __builtin_amdgcn_classf(x, kClassNaN) || !(a < p.thr);
    return keep ? bits : res;
}

// The same for inputs that are all finite and a saturating plan (a block whose largest magnitude
// is finite): no NaN, nothing at or above thr = +Inf, so nothing is returned unchanged.
// Round to nearest even with an anchor A = 2^(q+23): the clamped magnitude a is at most
// 2^(q+wl-1) <= A, so a + A lies in [A, 2A], where fp32 numbers are spaced 2^q apart: the addition
// itself rounds a to the nearest multiple of 2^q, ties to the even multiple (A / 2^q is even), and
// taking A away again is exact.  Two additions instead of scale, round, scale back.
template <int MODE>
__device__ __forceinline__ uint32_t quantize_finite_to_grid(uint32_t bits, const GridPlan& p, uint32_t r)
{
    const float x = __uint_as_float(bits);
    const float a = __builtin_fabsf(__builtin_amdgcn_fmed3f(x, p.lo, p.hi));
    float v;
    if (MODE == QSIM_RN_EVEN) {
        float sum = a + p.anchor;
        asm("" : "+v"(sum));                        // (the two additions must stay two additions)
        v = sum - p.anchor;
    } else {
        v = __builtin_ldexpf(round_scaled<MODE>(__builtin_ldexpf(a, -p.q), r), p.q);
    }
    return (__float_as_uint(v) & 0x7fffffffu) | (bits & 0x80000000u);
}

// Whether quantize_finite_to_grid may stand in for quantize_to_grid under this plan.
template <int MODE>
__device__ __forceinline__ bool plan_is_finite(const GridPlan& p)
{
    return MODE == QSIM_RN_EVEN ? p.anchor != 0.0f : p.finite != 0;
}

// Grid plan of a block from the largest magnitude encoding found in it.
__device__ __forceinline__ GridPlan block_plan(uint32_t max_mag, int wl, int symmetric)
{
    uint32_t field = max_mag >> 23;
    field = field < 1u ? 1u : (field > 254u ? 254u : field);
    GridPlan p;
    p.q = (int)field - 125 - wl;                     // e_s + 2 - wl
    // Kmax * 2^q = 2^(e_s+1) - 2^q: exponent field of e_s with the top wl-2 fraction bits set
    const uint32_t pos = (field << 23) | (((1u << (wl - 2)) - 1u) << (25 - wl));
    const uint32_t neg = symmetric ? pos : ((field + 1u) << 23);      // 2^(e_s+1), Inf when e_s = 127
    p.hi = __uint_as_float(pos);
    p.lo = __uint_as_float(neg | 0x80000000u);
    p.thr = __builtin_inff();
    p.finite = max_mag < 0x7f800000u ? 1 : 0;
    const int anchor_field = p.q + 23 + 127;         // at least 2: q >= 1 - 125 - 24
    p.anchor = p.finite && anchor_field <= 254 ? __uint_as_float((uint32_t)anchor_field << 23) : 0.0f;
    return p;
}

// The same plan for kernels that keep a table of blocks and take a plan per element: every constant
// of the plan is f23 = (exponent field of the block's largest magnitude, clamped to 1..254) << 23
// with a constant of the format or'ed or added in, so the table holds f23 and a plan costs three
// operations.  Only for blocks for which plan_is_finite holds (the anchor exists, nothing is NaN).
struct FieldPlan {
    uint32_t hi_or;        // the top wl - 2 fraction bits
    uint32_t lo_add;       // sign and: the same bits (symmetric), or one more in the exponent field
    uint32_t anchor_add;   // (25 - wl) << 23
    int q_add;             // -125 - wl
};

__device__ __forceinline__ FieldPlan field_plan(int wl, int symmetric)
{
    FieldPlan c;
    c.hi_or = ((1u << (wl - 2)) - 1u) << (25 - wl);
    c.lo_add = 0x80000000u + (symmetric ? c.hi_or : 0x00800000u);
    c.anchor_add = (uint32_t)(25 - wl) << 23;
    c.q_add = -125 - wl;
    return c;
}

__device__ __forceinline__ uint32_t clamped_field23(uint32_t max_mag)
{
    const uint32_t field = max_mag >> 23;
    return (field < 1u ? 1u : (field > 254u ? 254u : field)) << 23;
}

__device__ __forceinline__ GridPlan plan_of_field(uint32_t f23, const FieldPlan& c)
{
    GridPlan p;
    p.q = (int)(f23 >> 23) + c.q_add;
    p.hi = __uint_as_float(f23 | c.hi_or);
    p.lo = __uint_as_float(f23 + c.lo_add);
    p.thr = __builtin_inff();
    p.anchor = __uint_as_float(f23 + c.anchor_add);
    p.finite = 1;
    return p;
}

// ---------------------------------------------------------------------------------------------
// Custom floating point (Sec. 3.1 "Number Formats", first paragraph).  As above, one code path per
// form; saturation and flushing are constants of the plan:
//   max_enc     encoding of the largest value, or of Inf when the format does not saturate
//   keep_thr    magnitude encodings from here on are returned unchanged: NaN (0x7f800001) when the
//               format saturates, Inf and NaN (0x7f800000) when it does not
//   min_normal  encoding of 2^emin when results below it are flushed to zero, else 0
//
// "Shift" form: every input that is not flushed loses the same `drop` = 23 - M low fraction bits,
// so rounding is integer arithmetic on the encoding with a constant mask; a carry runs into the
// exponent field by itself.  Valid when the format has no binade of its own below fp32's (E = 8
// with gradual underflow: fp32 denormals share the step of the lowest binade) or when results
// below 2^emin are flushed.  With E = 8 and flushing (`denormal_inputs`), fp32 denormal inputs are
// rounded with their true exponent on a rarely taken side path, since the largest of them can
// round up to 2^-126 and survive.
// ---------------------------------------------------------------------------------------------
struct FloatPlan {
    int drop;             // 23 - man_bits
    int man_bits;
    int emin_field;       // emin + 127: exponent field of the smallest normal binade
    uint32_t max_enc;
    uint32_t keep_thr;
    uint32_t min_normal;
    int denormal_inputs;
};

template <int MODE>
__device__ __forceinline__ uint32_t round_encoding(uint32_t mag, int drop, uint32_t r)
{
    // rounds the magnitude encoding to a multiple of 2^drop units in the last place; 1 <= drop <= 22
    const uint32_t mask = (1u << drop) - 1u;
    uint32_t inc;
    if (MODE == QSIM_RN_EVEN) inc = (mask >> 1) + ((mag >> drop) & 1u);
    else if (MODE == QSIM_RN_AWAY) inc = (mask >> 1) + 1u;
    else if (MODE == QSIM_RN_ZERO) inc = mask >> 1;
    else inc = (r >> (32 - drop)) ^ mask;       // up  <=>  r < rem * 2^(32-drop)  <=>  rem + (mask - (r >> (32-drop))) > mask
    return (mag + inc) & ~mask;
}

// DENORMAL_INPUTS is a template parameter because the side path, once compiled in, is executed
// under a lane mask for every element (about 40 instructions per group), denormal or not.
template <int MODE, bool DENORMAL_INPUTS>
__device__ __forceinline__ uint32_t quantize_float_shift(uint32_t bits, const FloatPlan& p, uint32_t r)
{
    const uint32_t mag0 = bits & 0x7fffffffu;
    const uint32_t mag = mag0 < p.max_enc ? mag0 : p.max_enc;
    uint32_t res = p.drop ? round_encoding<MODE>(mag, p.drop, r) : mag;
    if (DENORMAL_INPUTS && mag - 1u < 0x7fffffu) {
        // fp32 denormal: keep man_bits below the leading one of the fraction
        const int top = 31 - __builtin_clz(mag);
        const int s = top - p.man_bits;
        res = s > 0 ? round_encoding<MODE>(mag, s, r) : mag;
    }
    res = res < p.min_normal ? 0u : res;
    res |= bits & 0x80000000u;
    return mag0 >= p.keep_thr ? bits : res;
}

// "General" form, gradual underflow with E < 8: the grid step depends on the element,
// 2^(max(e, emin) - M); scale by it, round, scale back.  y < 2^(M+1) <= 2^24.
template <int MODE>
__device__ __forceinline__ uint32_t quantize_float_general(uint32_t bits, const FloatPlan& p, uint32_t r)
{
    const uint32_t mag0 = bits & 0x7fffffffu;
    const uint32_t mag = mag0 < p.max_enc ? mag0 : p.max_enc;
    const float a = __uint_as_float(mag);
    int field = (int)(mag >> 23);
    field = field > p.emin_field ? field : p.emin_field;
    const int q = field - 127 - p.man_bits;
    const float y = __builtin_ldexpf(a, -q);
    const float v = __builtin_ldexpf(round_scaled<MODE>(y, r), q);
    const uint32_t res = (__float_as_uint(v) & 0x7fffffffu) | (bits & 0x80000000u);
    return mag0 >= p.keep_thr ? bits : res;
}

// ---------------------------------------------------------------------------------------------
// A format chosen at run time (wave-uniform branches): used by the fused SGD step and by the
// dword path for arrays that are not 16-byte aligned.
// ---------------------------------------------------------------------------------------------
enum { kFloatShift = 0, kFloatGeneral = 1 };

struct FormatPlan {
    int kind;           // qsim_format::kind
    int mode;           // rounding
    int float_form;     // kFloatShift or kFloatGeneral
    int wl;             // block: word length
    int symmetric;      // block: symmetric clamp
    int lanes;          // block: lanes (groups of 4 elements) per chunk = L / 4
    GridPlan grid;      // fixed
    FloatPlan flt;      // float
};

template <int MODE>
__device__ __forceinline__ uint4 quantize_group_mode(const FormatPlan& f, const GridPlan& grid, const uint4& v, const Words4& r)
{
    uint4 o;
    if (f.kind == 1) {
        if (f.float_form == kFloatGeneral) {
            o.x = quantize_float_general<MODE>(v.x, f.flt, r.w[0]);
            o.y = quantize_float_general<MODE>(v.y, f.flt, r.w[1]);
            o.z = quantize_float_general<MODE>(v.z, f.flt, r.w[2]);
            o.w = quantize_float_general<MODE>(v.w, f.flt, r.w[3]);
        } else if (f.flt.denormal_inputs) {
            o.x = quantize_float_shift<MODE, true>(v.x, f.flt, r.w[0]);
            o.y = quantize_float_shift<MODE, true>(v.y, f.flt, r.w[1]);
            o.z = quantize_float_shift<MODE, true>(v.z, f.flt, r.w[2]);
            o.w = quantize_float_shift<MODE, true>(v.w, f.flt, r.w[3]);
        } else {
            o.x = quantize_float_shift<MODE, false>(v.x, f.flt, r.w[0]);
            o.y = quantize_float_shift<MODE, false>(v.y, f.flt, r.w[1]);
            o.z = quantize_float_shift<MODE, false>(v.z, f.flt, r.w[2]);
            o.w = quantize_float_shift<MODE, false>(v.w, f.flt, r.w[3]);
        }
    } else {
        o.x = quantize_to_grid<MODE>(v.x, grid, r.w[0]);
        o.y = quantize_to_grid<MODE>(v.y, grid, r.w[1]);
        o.z = quantize_to_grid<MODE>(v.z, grid, r.w[2]);
        o.w = quantize_to_grid<MODE>(v.w, grid, r.w[3]);
    }
    return o;
}

// Quantize the four elements of a group with a float format, or with the given grid (fixed point,
// or a block's plan), the rounding mode chosen at run time.
__device__ __forceinline__ uint4 quantize_group_rt(const FormatPlan& f, const GridPlan& grid, const uint4& v, const Words4& r)
{
    switch (f.mode) {
    case QSIM_RN_EVEN: return quantize_group_mode<QSIM_RN_EVEN>(f, grid, v, r);
    case QSIM_RN_AWAY: return quantize_group_mode<QSIM_RN_AWAY>(f, grid, v, r);
    case QSIM_RN_ZERO: return quantize_group_mode<QSIM_RN_ZERO>(f, grid, v, r);
    default:           return quantize_group_mode<QSIM_STOCHASTIC>(f, grid, v, r);
    }
}

// ---------------------------------------------------------------------------------------------
// Wavefront maximum of an unsigned value: DPP butterflies inside each row of 16 lanes, one
// ds_swizzle across the two rows of a half, then the two halves through scalar reads.
// ---------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max(uint32_t v)
{
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
    return v > o ? v : o;
}

// Maximum over aligned groups of `lanes` consecutive lanes (a power of two, 1..64); every lane of
// a group receives the group's maximum.
__device__ __forceinline__ uint32_t group_max(uint32_t v, int lanes)
{
    if (lanes >= 2)  v = dpp_max<0xB1>(v);     // quad_perm [1,0,3,2]: lane ^ 1
    if (lanes >= 4)  v = dpp_max<0x4E>(v);     // quad_perm [2,3,0,1]: lane ^ 2
    if (lanes >= 8)  v = dpp_max<0x141>(v);    // row_half_mirror: joins the two quads of each 8
    if (lanes >= 16) v = dpp_max<0x140>(v);    // row_mirror: joins the two halves of a row
    if (lanes >= 32) {
        const uint32_t o = (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F);   // lane ^ 16
        v = v > o ? v : o;
    }
    if (lanes >= 64) {
        const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
        const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
        v = a > b ? a : b;
    }
    return v;
}

// Maximum over the whole wavefront; the result is wave-uniform.
__device__ __forceinline__ uint32_t wave_max(uint32_t v) { return group_max(v, 64); }

__device__ __forceinline__ uint32_t max4_mag(const uint4& b)
{
    const uint32_t a0 = b.x & 0x7fffffffu, a1 = b.y & 0x7fffffffu;
    const uint32_t a2 = b.z & 0x7fffffffu, a3 = b.w & 0x7fffffffu;
    const uint32_t m0 = a0 > a1 ? a0 : a1, m1 = a2 > a3 ? a2 : a3;
    return m0 > m1 ? m0 : m1;
}

}  // namespace qsim
