"""Independent brute-force models of the formats, used only to pin the oracle.

Nothing here is derived from the oracle's code: a format is described by the SET of values it can
represent, enumerated explicitly, and rounding is "pick a neighbour from the set" in exact
rational arithmetic.
"""
from __future__ import annotations

import bisect
from fractions import Fraction

import numpy as np

RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC = 0, 1, 2, 3
SATURATE, SUBNORMAL, SYMMETRIC = 1, 2, 4


def f32_to_fraction(x) -> Fraction:
    return Fraction(float(np.float32(x)))


def float_value_set(exp_bits: int, man_bits: int, subnormal: bool, lo_exp: int = -175, hi_exp: int = 131):
    """Sorted non-negative values of float(E, M) with the exponent range left open at both ends
    (the range rules are applied afterwards), as (values, is_even_code) lists.

    With gradual underflow the values below 2^emin are the multiples of 2^(emin - M)."""
    bias = (1 << (exp_bits - 1)) - 1
    emin = 1 - bias
    vals = {}
    first_exp = emin if subnormal else lo_exp
    for e in range(first_exp, hi_exp + 1):
        for m in range(1 << man_bits):
            vals[Fraction(2) ** e * (1 + Fraction(m, 1 << man_bits))] = (m % 2 == 0)
    if subnormal:
        for m in range(1 << man_bits):
            vals[Fraction(2) ** emin * Fraction(m, 1 << man_bits)] = (m % 2 == 0)
    else:
        vals[Fraction(0)] = True
    keys = sorted(vals)
    return keys, [vals[k] for k in keys]


def pick_neighbour(a: Fraction, keys, even, rounding: int, r: int):
    """Round the non-negative rational a to a member of the sorted set `keys`."""
    i = bisect.bisect_right(keys, a) - 1
    lo = keys[i]
    if lo == a:
        return lo
    hi = keys[i + 1]
    f = (a - lo) / (hi - lo)
    if rounding == STOCHASTIC:
        t = (f * (1 << 32)).__floor__()
        return hi if r < t else lo
    if f > Fraction(1, 2):
        return hi
    if f < Fraction(1, 2):
        return lo
    if rounding == RN_AWAY:
        return hi
    if rounding == RN_ZERO:
        return lo
    return lo if even[i] else hi


def model_float(x, exp_bits, man_bits, rounding, flags, r, sets_cache={}):
    x = np.float32(x)
    if np.isnan(x) or x == 0:
        return x
    bias = (1 << (exp_bits - 1)) - 1
    emin = 1 - bias
    maxval = (2 - Fraction(1, 1 << man_bits)) * Fraction(2) ** bias
    if np.isinf(x):
        return np.float32(np.copysign(float(maxval), x)) if flags & SATURATE else x
    key = (exp_bits, man_bits, bool(flags & SUBNORMAL))
    if key not in sets_cache:
        sets_cache[key] = float_value_set(*key)
    keys, even = sets_cache[key]
    a = abs(f32_to_fraction(x))
    if not (flags & SUBNORMAL) and a < keys[1]:
        v = Fraction(0)                       # far below anything a format can hold
    else:
        v = pick_neighbour(a, keys, even, rounding, r)
    if not (flags & SUBNORMAL) and v < Fraction(2) ** emin:
        v = Fraction(0)
    if (flags & SATURATE) and v > maxval:
        v = maxval
    out = float(v)
    if out > float(np.finfo(np.float32).max):
        out = float("inf")
    return np.float32(np.copysign(out, x))


def model_fixed(x, wl, fl, rounding, flags, r):
    """Fixed point by its value set: the integers K times 2^-fl."""
    x = np.float32(x)
    if np.isnan(x):
        return x
    step = Fraction(2) ** (-fl)
    kmax = (1 << (wl - 1)) - 1
    kmin = -kmax if flags & SYMMETRIC else -(1 << (wl - 1))
    if np.isinf(x):
        if not flags & SATURATE:
            return x
        return np.float32(float((kmax if x > 0 else kmin) * step))
    a = abs(f32_to_fraction(x)) / step
    k = a.__floor__()
    f = a - k
    if rounding == STOCHASTIC:
        up = r < (f * (1 << 32)).__floor__()
    elif f != Fraction(1, 2):
        up = f > Fraction(1, 2)
    else:
        up = {RN_AWAY: True, RN_ZERO: False, RN_EVEN: k % 2 == 1}[rounding]
    K = k + (1 if up else 0)
    Ks = -K if np.signbit(x) else K
    if flags & SATURATE:
        Ks = max(kmin, min(kmax, Ks))
    out = float(abs(Ks) * step)
    if out > float(np.finfo(np.float32).max):
        out = float("inf")
    return np.float32(np.copysign(out, x))


def round_fraction_to_f32(v: Fraction) -> np.float32:
    """Correctly rounded (nearest even) fp32 of an exact rational; finite range only."""
    if v == 0:
        return np.float32(0.0)
    s = -1 if v < 0 else 1
    a = abs(v)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    e = max(e, -126)
    ulp = Fraction(2) ** (e - 23)
    y = a / ulp
    k = y.__floor__()
    f = y - k
    if f > Fraction(1, 2) or (f == Fraction(1, 2) and k % 2 == 1):
        k += 1
    return np.float32(s * float(k * ulp))


def bits(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def assert_bit_equal(got, want, what=""):
    g, w = bits(got).reshape(-1), bits(want).reshape(-1)
    assert g.shape == w.shape, (g.shape, w.shape)
    bad = np.nonzero(g != w)[0]
    if bad.size:
        i = int(bad[0])
        raise AssertionError(
            f"{what}: {bad.size} of {g.size} elements differ; first at {i}: "
            f"got 0x{int(g[i]):08x} ({np.float32(g[i:i+1].view(np.float32)[0])!r}) "
            f"want 0x{int(w[i]):08x} ({np.float32(w[i:i+1].view(np.float32)[0])!r})")
