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

struct RngKey {
    uint32_t seed_lo, seed_hi, stream_id;
};

// Random words of the four elements 4*j .. 4*j+3 (Sec. 3.1 "Rounding mode": stochastic rounding).
__device__ __forceinline__ Words4 random_words(uint64_t j, const RngKey& key, uint32_t role)
{
    return philox4x32_10((uint32_t)j, (uint32_t)(j >> 32), key.stream_id, role, key.seed_lo, key.seed_hi);
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
// y = |x| / 2^q is at most 2^23.  Without saturation, inputs of 2^(q+24) and above are already on
// the grid and are returned as they are (so are NaN and Inf, which fail the same comparison).
// A y that underflows fp32 is below 2^-126: it rounds to zero in every mode either way.
// ---------------------------------------------------------------------------------------------
struct GridPlan {
    int q;                // grid step 2^q
    float lo, hi;         // saturating: most negative and largest value (grid points)
    float thr;            // not saturating: 2^(q+24), or +Inf when that is beyond fp32
    uint32_t keep_class;  // saturating: v_cmp_class mask of inputs returned unchanged (NaN; -Inf when lo is -Inf)
};

constexpr uint32_t kClassNaN = 0x003u;
constexpr uint32_t kClassNegInf = 0x004u;

template <int MODE, bool SAT>
__device__ __forceinline__ uint32_t quantize_to_grid(uint32_t bits, const GridPlan& p, uint32_t r)
{
    const float x = __uint_as_float(bits);
    const float a = SAT ? __builtin_fabsf(__builtin_amdgcn_fmed3f(x, p.lo, p.hi)) : __builtin_fabsf(x);
    const float y = __builtin_ldexpf(a, -p.q);
    const float v = __builtin_ldexpf(round_scaled<MODE>(y, r), p.q);
    const uint32_t res = (__float_as_uint(v) & 0x7fffffffu) | (bits & 0x80000000u);
    const bool keep = SAT ? __builtin_amdgcn_classf(x, (int)p.keep_class) : !(a < p.thr);
    return keep ? bits : res;
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
    p.thr = 0.0f;
    p.keep_class = kClassNaN | (neg == 0x7f800000u ? kClassNegInf : 0u);
    return p;
}

// ---------------------------------------------------------------------------------------------
// Custom floating point (Sec. 3.1 "Number Formats", first paragraph).
//
// "Shift" form: every input that is not flushed loses the same `drop` = 23 - M low fraction bits,
// so rounding is integer arithmetic on the encoding with a constant mask; a carry runs into the
// exponent field by itself.  Valid when the format has no binade of its own below fp32's (E = 8
// with gradual underflow: fp32 denormals share the step of the lowest binade) or when results
// below 2^emin are flushed.  FTZ = 1: flush.  FTZ = 2: flush, and fp32 denormal inputs (possible
// survivors only when E = 8) are rounded with their true exponent on a rarely taken side path.
// ---------------------------------------------------------------------------------------------
struct FloatPlan {
    int drop;             // 23 - man_bits
    int man_bits;
    int emin_field;       // emin + 127: exponent field of the smallest normal binade
    uint32_t max_enc;     // encoding of the largest value
    uint32_t min_normal;  // encoding of 2^emin
    float maxval;         // the largest value
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

template <int MODE, bool SAT, int FTZ>
__device__ __forceinline__ uint32_t quantize_float_shift(uint32_t bits, const FloatPlan& p, uint32_t r)
{
    const uint32_t mag0 = bits & 0x7fffffffu;
    const uint32_t mag = SAT ? (mag0 < p.max_enc ? mag0 : p.max_enc) : mag0;      // Inf saturates; without SAT it stays Inf below
    uint32_t res = p.drop ? round_encoding<MODE>(mag, p.drop, r) : mag;
    if (FTZ == 2 && mag - 1u < 0x7fffffu) {
        // fp32 denormal: keep man_bits below the leading one of the fraction
        const int top = 31 - __builtin_clz(mag);
        const int s = top - p.man_bits;
        res = s > 0 ? round_encoding<MODE>(mag, s, r) : mag;
    }
    if (FTZ) res = res < p.min_normal ? 0u : res;
    res |= bits & 0x80000000u;
    return mag0 > 0x7f800000u ? bits : res;                                     // NaN passes through
}

// "General" form, gradual underflow with E < 8: the grid step depends on the element,
// 2^(max(e, emin) - M); scale by it, round, scale back.  y < 2^(M+1) <= 2^24.
template <int MODE, bool SAT>
__device__ __forceinline__ uint32_t quantize_float_general(uint32_t bits, const FloatPlan& p, uint32_t r)
{
    const float x = __uint_as_float(bits);
    const float a = SAT ? __builtin_fminf(__builtin_fabsf(x), p.maxval) : __builtin_fabsf(x);
    int field = (int)(__float_as_uint(a) >> 23);
    field = field > p.emin_field ? field : p.emin_field;
    const int q = field - 127 - p.man_bits;
    const float y = __builtin_ldexpf(a, -q);
    const float v = __builtin_ldexpf(round_scaled<MODE>(y, r), q);
    const uint32_t res = (__float_as_uint(v) & 0x7fffffffu) | (bits & 0x80000000u);
    // NaN always passes; Inf passes unless it saturated to maxval above
    const bool keep = SAT ? (x != x) : !(a < __builtin_inff());
    return keep ? bits : res;
}

// ---------------------------------------------------------------------------------------------
// A format chosen at run time (wave-uniform branches): used by the fused SGD step and by the
// dword path for arrays that are not 16-byte aligned.
// ---------------------------------------------------------------------------------------------
enum { kFloatShift = 0, kFloatGeneral = 1 };

struct FormatPlan {
    int kind;           // qsim_format::kind
    int mode;           // rounding
    int saturate;       // float / fixed
    int float_form;     // kFloatShift or kFloatGeneral
    int ftz;            // shift form: 0, 1, 2 as above
    int wl;             // block: word length
    int symmetric;      // block: symmetric clamp
    int lanes;          // block: lanes (groups of 4 elements) per chunk = L / 4
    GridPlan grid;      // fixed
    FloatPlan flt;      // float
};

template <int MODE>
__device__ __forceinline__ uint32_t quantize_float_rt(const FormatPlan& f, uint32_t bits, uint32_t r)
{
    if (f.float_form == kFloatGeneral)
        return f.saturate ? quantize_float_general<MODE, true>(bits, f.flt, r)
                          : quantize_float_general<MODE, false>(bits, f.flt, r);
    if (f.saturate) {
        if (f.ftz == 0) return quantize_float_shift<MODE, true, 0>(bits, f.flt, r);
        if (f.ftz == 1) return quantize_float_shift<MODE, true, 1>(bits, f.flt, r);
        return quantize_float_shift<MODE, true, 2>(bits, f.flt, r);
    }
    if (f.ftz == 0) return quantize_float_shift<MODE, false, 0>(bits, f.flt, r);
    if (f.ftz == 1) return quantize_float_shift<MODE, false, 1>(bits, f.flt, r);
    return quantize_float_shift<MODE, false, 2>(bits, f.flt, r);
}

template <int MODE>
__device__ __forceinline__ uint32_t quantize_grid_rt(int saturate, const GridPlan& p, uint32_t bits, uint32_t r)
{
    return saturate ? quantize_to_grid<MODE, true>(bits, p, r) : quantize_to_grid<MODE, false>(bits, p, r);
}

// Quantize the four elements of a group with a float or fixed format chosen at run time.
__device__ __forceinline__ uint4 quantize_group_rt(const FormatPlan& f, const GridPlan& grid, int grid_saturate,
                                                   const uint4& v, const Words4& r)
{
    uint4 o;
#define QSIM_APPLY4(EXPR_X, EXPR_Y, EXPR_Z, EXPR_W) \
    do { o.x = EXPR_X; o.y = EXPR_Y; o.z = EXPR_Z; o.w = EXPR_W; } while (0)
#define QSIM_BY_MODE(FN, ...)                                                                                   \
    switch (f.mode) {                                                                                           \
    case QSIM_RN_EVEN:                                                                                          \
        QSIM_APPLY4(FN<QSIM_RN_EVEN>(__VA_ARGS__, v.x, r.w[0]), FN<QSIM_RN_EVEN>(__VA_ARGS__, v.y, r.w[1]),     \
                    FN<QSIM_RN_EVEN>(__VA_ARGS__, v.z, r.w[2]), FN<QSIM_RN_EVEN>(__VA_ARGS__, v.w, r.w[3]));    \
        break;                                                                                                  \
    case QSIM_RN_AWAY:                                                                                          \
        QSIM_APPLY4(FN<QSIM_RN_AWAY>(__VA_ARGS__, v.x, r.w[0]), FN<QSIM_RN_AWAY>(__VA_ARGS__, v.y, r.w[1]),     \
                    FN<QSIM_RN_AWAY>(__VA_ARGS__, v.z, r.w[2]), FN<QSIM_RN_AWAY>(__VA_ARGS__, v.w, r.w[3]));    \
        break;                                                                                                  \
    case QSIM_RN_ZERO:                                                                                          \
        QSIM_APPLY4(FN<QSIM_RN_ZERO>(__VA_ARGS__, v.x, r.w[0]), FN<QSIM_RN_ZERO>(__VA_ARGS__, v.y, r.w[1]),     \
                    FN<QSIM_RN_ZERO>(__VA_ARGS__, v.z, r.w[2]), FN<QSIM_RN_ZERO>(__VA_ARGS__, v.w, r.w[3]));    \
        break;                                                                                                  \
    default:                                                                                                    \
        QSIM_APPLY4(FN<QSIM_STOCHASTIC>(__VA_ARGS__, v.x, r.w[0]), FN<QSIM_STOCHASTIC>(__VA_ARGS__, v.y, r.w[1]), \
                    FN<QSIM_STOCHASTIC>(__VA_ARGS__, v.z, r.w[2]), FN<QSIM_STOCHASTIC>(__VA_ARGS__, v.w, r.w[3])); \
        break;                                                                                                  \
    }
    if (f.kind == 1) {
        QSIM_BY_MODE(quantize_float_rt, f)
    } else {
        QSIM_BY_MODE(quantize_grid_rt, grid_saturate, grid)
    }
#undef QSIM_BY_MODE
#undef QSIM_APPLY4
    return o;
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
