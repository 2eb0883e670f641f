// Device-side building blocks: Philox4x32-10, bit-level rounding of the fp32 encoding to a
// power-of-two grid, the three format rules, and wavefront reductions.  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "qsim.h"

namespace qsim {

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  key and the two upper counter words are wave-uniform,
// so the key schedule lives in scalar registers; the 32x32->64 products map to v_mad_u64_u32.
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

// Random words of the four elements 4*j .. 4*j+3 (Sec. 3.1 "Rounding mode": stochastic rounding).
__device__ __forceinline__ Words4 random_words(uint64_t j, uint32_t seed_lo, uint32_t seed_hi,
                                               uint32_t stream_id, uint32_t role)
{
    return philox4x32_10((uint32_t)j, (uint32_t)(j >> 32), stream_id, role, seed_lo, seed_hi);
}

// ---------------------------------------------------------------------------------------------
// Rounding primitive on the encoding (Sec. 3.1 "Rounding mode").
//
// `mag` is the encoding of a finite magnitude (sign bit clear).  With significand integer m
// (24 bits, implicit one unless the exponent field is 0) and e1 = max(field, 1), |x| = m * 2^(e1-150).
// Rounding to a multiple of 2^q removes the s = q + 150 - e1 lowest bits of m:
//   s <= 0      x is already on the grid
//   1..23       the removed bits all sit in the fraction field; adding the carry to the encoding
//               propagates into the exponent field by itself
//   s >= 24     the whole significand is below the grid: the result is 0 or 2^q
// Returns the encoding of the rounded magnitude (0x7f800000 when it passes the fp32 range).
// Requires -126 <= q <= 127 whenever s >= 24 can occur with a non-zero result.
// ---------------------------------------------------------------------------------------------
template <int MODE>
__device__ __forceinline__ bool round_up_decision(uint32_t rem, uint32_t half, uint32_t odd, uint32_t t,
                                                  uint32_t r)
{
    if (MODE == QSIM_RN_EVEN) return rem > half || (rem == half && odd);
    if (MODE == QSIM_RN_AWAY) return rem >= half;
    if (MODE == QSIM_RN_ZERO) return rem > half;
    return r < t;
}

template <int MODE>
__device__ __forceinline__ uint32_t round_magnitude(uint32_t mag, int s, int q, uint32_t r)
{
    if (s <= 0) return mag;
    const uint32_t field = mag >> 23;
    const uint32_t m = (mag & 0x7fffffu) | (field ? 0x800000u : 0u);
    if (s <= 23) {
        const uint32_t mask = (1u << s) - 1u;
        const uint32_t rem = m & mask;
        const uint32_t half = 1u << (s - 1);
        const uint32_t odd = (m >> s) & 1u;
        const uint32_t t = rem << (32 - s);                 // floor(f * 2^32), exact
        const bool up = round_up_decision<MODE>(rem, half, odd, t, r);
        return (mag & ~mask) + (up ? (1u << s) : 0u);
    }
    // s >= 24: k = 0 (even), f = m / 2^s
    bool up;
    if (MODE == QSIM_STOCHASTIC) {
        const uint32_t t = (s <= 32) ? (m << (32 - s)) : ((s < 64) ? (m >> (s - 32)) : 0u);
        up = r < t;
    } else if (s == 24) {
        up = round_up_decision<MODE>(m, 0x800000u, 0u, 0u, 0u);
    } else {
        up = false;                                         // f < 1/2
    }
    return up ? ((uint32_t)(q + 127) << 23) : 0u;
}

// The same with the mode chosen at run time (wave-uniform branch).
__device__ __forceinline__ uint32_t round_magnitude_rt(int mode, uint32_t mag, int s, int q, uint32_t r)
{
    switch (mode) {
    case QSIM_RN_EVEN: return round_magnitude<QSIM_RN_EVEN>(mag, s, q, r);
    case QSIM_RN_AWAY: return round_magnitude<QSIM_RN_AWAY>(mag, s, q, r);
    case QSIM_RN_ZERO: return round_magnitude<QSIM_RN_ZERO>(mag, s, q, r);
    default:           return round_magnitude<QSIM_STOCHASTIC>(mag, s, q, r);
    }
}

// ---------------------------------------------------------------------------------------------
// Fixed-grid quantizer: fixed point, and block floating point once the shared exponent is known
// (Sec. 3.1 "Number Formats", second paragraph).  Both limits are grid points, rounding is
// monotone and leaves grid points alone, so clamping the INPUT magnitude to the limit gives the
// same result as clamping the rounded code.
// ---------------------------------------------------------------------------------------------
struct GridPlan {
    int q;             // grid step 2^q
    uint32_t pos_lim;  // encoding of the largest positive value, Kmax * 2^q
    uint32_t neg_lim;  // encoding of the magnitude of the most negative value
    int saturate;      // clamp to the limits (block formats always do)
};

template <int MODE>
__device__ __forceinline__ uint32_t quantize_to_grid(uint32_t bits, const GridPlan& p, uint32_t r)
{
    uint32_t mag = bits & 0x7fffffffu;
    const uint32_t sign = bits & 0x80000000u;
    if (mag > 0x7f800000u) return bits;                      // NaN passes through
    if (p.saturate) {
        const uint32_t lim = sign ? p.neg_lim : p.pos_lim;
        mag = mag < lim ? mag : lim;
    } else if (mag == 0x7f800000u) {
        return bits;
    }
    const uint32_t field = mag >> 23;
    const int s = p.q + 150 - (int)(field ? field : 1u);
    return sign | round_magnitude<MODE>(mag, s, p.q, r);
}

// Grid plan of a block from the largest magnitude encoding found in it.
__device__ __forceinline__ GridPlan block_plan(uint32_t max_mag, int wl, int symmetric)
{
    uint32_t field = max_mag >> 23;
    field = field < 1u ? 1u : (field > 254u ? 254u : field);
    GridPlan p;
    p.q = (int)field - 127 + 2 - wl;
    // Kmax * 2^q = 2^(e_s+1) - 2^q: exponent field of e_s with the top wl-2 fraction bits set
    p.pos_lim = (field << 23) | (((1u << (wl - 2)) - 1u) << (25 - wl));
    p.neg_lim = symmetric ? p.pos_lim : ((field + 1u) << 23);
    p.saturate = 1;
    return p;
}

// ---------------------------------------------------------------------------------------------
// Custom floating point (Sec. 3.1 "Number Formats", first paragraph).
// ---------------------------------------------------------------------------------------------
struct FloatPlan {
    int drop;            // 23 - man_bits: bits removed from a number in the format's normal range
    int man_bits;
    int emin_field;      // emin + 127: fp32 exponent field of the format's smallest normal binade
    uint32_t max_enc;    // encoding of the largest value
    uint32_t min_normal; // encoding of 2^emin
    int saturate;
    int subnormal;
};

template <int MODE>
__device__ __forceinline__ uint32_t quantize_float(uint32_t bits, const FloatPlan& p, uint32_t r)
{
    uint32_t mag = bits & 0x7fffffffu;
    const uint32_t sign = bits & 0x80000000u;
    if (mag > 0x7f800000u) return bits;
    if (p.saturate) {
        mag = mag < p.max_enc ? mag : p.max_enc;
    } else if (mag == 0x7f800000u) {
        return bits;
    }
    const int field = (int)(mag >> 23);
    const int e1 = field ? field : 1;
    uint32_t res;
    if (p.subnormal) {
        // grid step 2^(max(e, emin) - M); an fp32 denormal has e1 = 1 <= emin_field
        const int below = p.emin_field - e1;
        const int s = p.drop + (below > 0 ? below : 0);
        const int q = (below > 0 ? p.emin_field : e1) - 127 - p.man_bits;
        res = round_magnitude<MODE>(mag, s, q, r);
    } else {
        if (field) {
            res = round_magnitude<MODE>(mag, p.drop, field - 127 - p.man_bits, r);
        } else if (mag) {
            // fp32 denormal: true exponent from the leading one of the fraction
            const int top = 31 - __builtin_clz(mag);          // mag = frac, value frac * 2^-149
            const int s = top - p.man_bits;                   // keep man_bits below the leading one
            res = round_magnitude<MODE>(mag, s, top - 149 - p.man_bits, r);
        } else {
            res = 0u;
        }
        if (res < p.min_normal) res = 0u;                     // flush what stays below 2^emin
    }
    return sign | res;
}

// ---------------------------------------------------------------------------------------------
// Wavefront maximum of an unsigned value: DPP butterflies inside each row of 16 lanes, one
// ds_swizzle across the two rows of a half, then the two halves through scalar reads.
// The result is wave-uniform.
// ---------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max(uint32_t v)
{
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
    return v > o ? v : o;
}

__device__ __forceinline__ uint32_t row_max16(uint32_t v)
{
    v = dpp_max<0xB1>(v);    // quad_perm [1,0,3,2]: xor 1
    v = dpp_max<0x4E>(v);    // quad_perm [2,3,0,1]: xor 2
    v = dpp_max<0x141>(v);   // row_half_mirror: joins the two quads of each 8
    v = dpp_max<0x140>(v);   // row_mirror: joins the two halves of the row
    return v;
}

__device__ __forceinline__ uint32_t half_max32(uint32_t v)
{
    v = row_max16(v);
    const uint32_t o = (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F);   // lane ^ 16
    return v > o ? v : o;
}

__device__ __forceinline__ uint32_t wave_max(uint32_t v)
{
    v = half_max32(v);
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
    const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
    return a > b ? a : b;
}

// Maximum over aligned groups of `lanes` consecutive lanes (a power of two, 1..64); every lane of
// a group receives the group's maximum.
__device__ __forceinline__ uint32_t group_max(uint32_t v, int lanes)
{
    if (lanes >= 2)  v = dpp_max<0xB1>(v);
    if (lanes >= 4)  v = dpp_max<0x4E>(v);
    if (lanes >= 8)  v = dpp_max<0x141>(v);
    if (lanes >= 16) v = dpp_max<0x140>(v);
    if (lanes >= 32) {
        const uint32_t o = (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F);
        v = v > o ? v : o;
    }
    if (lanes >= 64) {
        const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
        const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
        v = a > b ? a : b;
    }
    return v;
}

__device__ __forceinline__ uint32_t max4_mag(const uint4& b)
{
    const uint32_t a0 = b.x & 0x7fffffffu, a1 = b.y & 0x7fffffffu;
    const uint32_t a2 = b.z & 0x7fffffffu, a3 = b.w & 0x7fffffffu;
    const uint32_t m0 = a0 > a1 ? a0 : a1, m1 = a2 > a3 ? a2 : a3;
    return m0 > m1 ? m0 : m1;
}

}  // namespace qsim
