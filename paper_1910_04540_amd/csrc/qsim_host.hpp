// Host-side argument validation and format plans shared by the entry points.  No HIP calls here:
// everything in this header runs before the first launch, so it is testable without a GPU.
#pragma once

#include <math.h>
#include <stdint.h>
#include <string.h>

#include "qsim.h"
#include "qsim_device.hpp"

namespace qsim {

constexpr uint64_t kMaxElements = 1ull << 38;   // keeps every grid below 2^31 workgroups

// Position of a shard's first element in the whole tensor: whole groups, and far from wrapping.
inline bool valid_index0(uint64_t index0) { return index0 % 4 == 0 && index0 <= (1ull << 62); }
inline bool valid_rounding(int r) { return r >= QSIM_RN_EVEN && r <= QSIM_STOCHASTIC; }
inline bool valid_flags(uint32_t f) { return (f & ~(QSIM_SATURATE | QSIM_SUBNORMAL | QSIM_SYMMETRIC)) == 0; }
// Block quantize also takes the flag that says whose the scratch is.
inline bool valid_block_flags(uint32_t f) { return valid_flags(f & ~(uint32_t)QSIM_WORKSPACE_KEPT); }
inline bool valid_fixed(int wl, int fl) { return wl >= 1 && wl <= 24 && fl >= wl - 128 && fl <= 149; }
inline bool valid_float(int e, int m) { return e >= 2 && e <= 8 && m >= 1 && m <= 23; }
inline bool valid_block_wl(int wl) { return wl >= 2 && wl <= 24; }

// Byte ranges of n floats at a and b overlap without being the same range.
inline bool partial_overlap(const void* a, const void* b, uint64_t n)
{
    const uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b, len = (uintptr_t)n * 4u;
    if (pa == pb) return false;
    return pa < pb ? (pb - pa < len) : (pa - pb < len);
}
inline bool any_overlap(const void* a, const void* b, uint64_t n) { return a == b || partial_overlap(a, b, n); }

// Byte ranges [a, a + bytes_a) and [b, b + bytes_b) share at least one byte.
inline bool ranges_overlap(const void* a, uint64_t bytes_a, const void* b, uint64_t bytes_b)
{
    const uintptr_t pa = (uintptr_t)a, pb = (uintptr_t)b;
    return pa < pb + bytes_b && pb < pa + bytes_a;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

inline uint32_t float_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return u;
}

inline float bits_float(uint32_t u)
{
    float f;
    memcpy(&f, &u, 4);
    return f;
}

inline GridPlan fixed_plan(int wl, int fl, uint32_t flags)
{
    GridPlan p;
    p.q = -fl;
    if (flags & QSIM_SATURATE) {
        const double kmax = ldexp(1.0, wl - 1) - 1.0;
        const double kneg = (flags & QSIM_SYMMETRIC) ? kmax : ldexp(1.0, wl - 1);
        p.hi = (float)ldexp(kmax, p.q);               // exact: at most 23 significant bits
        p.lo = -(float)ldexp(kneg, p.q);
        p.thr = INFINITY;
    } else {
        p.hi = INFINITY;
        p.lo = -INFINITY;
        p.thr = (p.q + 24 <= 127) ? (float)ldexp(1.0, p.q + 24) : INFINITY;
    }
    p.anchor = 0.0f;                                  // inputs of an elementwise call may be anything
    p.finite = 0;
    return p;
}

// Float plan and the device form that carries it out.
inline FloatPlan float_plan(int exp_bits, int man_bits, uint32_t flags, int* form)
{
    FloatPlan p;
    const int bias = (1 << (exp_bits - 1)) - 1;
    const int emin = 1 - bias;
    const bool saturate = (flags & QSIM_SATURATE) != 0;
    const bool subnormal = (flags & QSIM_SUBNORMAL) != 0;
    p.drop = 23 - man_bits;
    p.man_bits = man_bits;
    p.emin_field = emin + 127;
    p.max_enc = saturate ? float_bits((float)ldexp(2.0 - ldexp(1.0, -man_bits), bias)) : 0x7f800000u;
    p.keep_thr = saturate ? 0x7f800001u : 0x7f800000u;
    p.min_normal = subnormal ? 0u : ((uint32_t)p.emin_field << 23);
    p.denormal_inputs = (!subnormal && exp_bits == 8) ? 1 : 0;
    *form = (subnormal && exp_bits < 8) ? kFloatGeneral : kFloatShift;
    return p;
}

// n must fit the [outer, nblocks, inner] view; only outer == 1 may leave the last block short.
inline bool valid_block_shape(uint64_t n, uint64_t outer, uint64_t nblocks, uint64_t inner)
{
    if (outer == 0 || nblocks == 0 || inner == 0) return false;
    const unsigned __int128 total = (unsigned __int128)outer * nblocks * inner;
    if (total > (unsigned __int128)kMaxElements * 4) return false;
    if (outer == 1) return n <= (uint64_t)total && n > (nblocks - 1) * inner;
    return n == (uint64_t)total;
}

// Resolves the format of one number category of the SGD step for the device.
inline int make_format_plan(const qsim_format* f, FormatPlan* out)
{
    if (!f) return QSIM_ERR_NULL;
    if (!valid_rounding(f->rounding)) return QSIM_ERR_ROUNDING;
    if (!valid_flags(f->flags)) return QSIM_ERR_FORMAT;
    FormatPlan p;
    memset(&p, 0, sizeof(p));
    p.kind = f->kind;
    p.mode = f->rounding;
    switch (f->kind) {
    case 0: break;
    case 1:
        if (!valid_float(f->a, f->b)) return QSIM_ERR_FORMAT;
        p.flt = float_plan(f->a, f->b, f->flags, &p.float_form);
        break;
    case 2:
        if (!valid_fixed(f->a, f->b)) return QSIM_ERR_FORMAT;
        p.grid = fixed_plan(f->a, f->b, f->flags);
        break;
    case 3:
        if (!valid_block_wl(f->a) || f->b < 4 || f->b > 1024 || (f->b & (f->b - 1)) != 0) return QSIM_ERR_FORMAT;
        p.wl = f->a;
        p.symmetric = (f->flags & QSIM_SYMMETRIC) ? 1 : 0;
        p.lanes = f->b / 4;
        break;
    default: return QSIM_ERR_FORMAT;
    }
    *out = p;
    return QSIM_OK;
}

}  // namespace qsim
