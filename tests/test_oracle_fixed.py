"""Pins for the oracle's fixed-point quantizer (Sec. 3.1 "Number Formats", "Rounding mode")."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import qsim_ref as R
from paper_1910_04540_amd import workloads as W
from helpers import (RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC, SATURATE, SYMMETRIC, model_fixed,
                     assert_bit_equal, f32_to_fraction)


def _spot_rows(golden_dir, kind):
    with open(os.path.join(golden_dir, "spot_values.txt")) as fh:
        for line in fh:
            t = line.split()
            if t and t[0] == kind:
                yield t[1:]


def test_spot_values(golden_dir):
    rows = list(_spot_rows(golden_dir, "fixed"))
    assert len(rows) >= 15
    for wl, fl, rounding, flags, x, want in rows:
        got = R.fixed_scalar(float(x), int(wl), int(fl), int(rounding), int(flags))
        assert float(got) == float(want), (wl, fl, rounding, flags, x, got, want)


def _closed_form(x, wl, fl, rounding, saturate=True):
    """Library-routine form: scale, round with numpy's rint / floor / ceil, clamp, scale back."""
    y = np.ldexp(x.astype(np.float64), fl)
    a = np.abs(y)
    if rounding == RN_EVEN:
        k = np.rint(a)                      # IEEE round-half-even
    elif rounding == RN_AWAY:
        k = np.floor(a + 0.5)
    else:
        k = np.ceil(a - 0.5)
    k = np.copysign(k, y)
    if saturate:
        k = np.clip(k, -(2.0 ** (wl - 1)), 2.0 ** (wl - 1) - 1)
    return np.copysign(np.abs(np.ldexp(k, -fl)), x).astype(np.float32)


@pytest.mark.parametrize("wl,fl", [(8, 6), (16, 12), (4, 0), (24, 20), (2, 1), (12, -3), (1, 0)])
@pytest.mark.parametrize("rounding", [RN_EVEN, RN_AWAY, RN_ZERO])
def test_nearest_equals_library_rounding(wl, fl, rounding):
    g = np.random.Generator(np.random.PCG64(21))
    step = 2.0 ** -fl
    x = np.concatenate([
        W.uniform_with_outliers(20000, seed=2) * np.float32(step * 2 ** (wl - 3)),
        # exact grid points, midpoints and their fp32 neighbours
        (np.arange(-300, 300) * step * 0.5).astype(np.float32),
        np.nextafter((np.arange(-300, 300) * step * 0.5).astype(np.float32), np.float32(np.inf)),
        np.nextafter((np.arange(-300, 300) * step * 0.5).astype(np.float32), np.float32(-np.inf)),
        (g.standard_normal(5000) * step).astype(np.float32),
        np.array([0.0, -0.0], dtype=np.float32),
    ])
    for sat in (True, False):
        got = R.fixed_quantize(x, wl, fl, rounding, SATURATE if sat else 0)
        assert_bit_equal(got, _closed_form(x, wl, fl, rounding, sat), f"fixed({wl},{fl}) mode {rounding} sat {sat}")


@pytest.mark.parametrize("wl,fl", [(4, 2), (6, 3), (3, -1), (5, 7)])
@pytest.mark.parametrize("flags", [0, SATURATE, SATURATE | SYMMETRIC])
def test_tiny_formats_by_value_set(wl, fl, flags):
    """Every mode, stochastic included, against the explicit value-set model in exact rationals."""
    g = np.random.Generator(np.random.PCG64(22))
    step = 2.0 ** -fl
    xs = np.concatenate([
        (g.uniform(-1.5, 1.5, 300) * step * 2 ** (wl - 1)).astype(np.float32),
        (np.arange(-40, 40) * step * 0.5).astype(np.float32),
        np.array([0.0, -0.0, np.inf, -np.inf, 1e30, -1e30, 1e-30, 1e-45], dtype=np.float32),
    ])
    rs = g.integers(0, 1 << 32, size=xs.size, dtype=np.uint64)
    for rounding in (RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC):
        for x, r in zip(xs, rs):
            got = R.fixed_scalar(x, wl, fl, rounding, flags, int(r))
            want = model_fixed(x, wl, fl, rounding, flags, int(r))
            assert got.view(np.uint32) == want.view(np.uint32), (x, rounding, flags, r, got, want)


def test_stochastic_threshold_is_exact():
    """up  <=>  r < floor(f * 2^32): checked at the threshold itself with hand-picked words."""
    wl, fl = 8, 6
    for x in (0.3, 1.0 / 3.0, 0.0078125, 1.9, 2.0 ** -20, 0.015625 + 2.0 ** -30, -0.7):
        x = np.float32(x)
        y = abs(f32_to_fraction(x)) * 64
        k = y.__floor__()
        t = ((y - k) * (1 << 32)).__floor__()
        lo = np.float32(np.copysign(k / 64.0, x))
        hi = np.float32(np.copysign((k + 1) / 64.0, x))
        if t > 0:
            assert R.fixed_scalar(x, wl, fl, STOCHASTIC, SATURATE, t - 1) == hi
            assert R.fixed_scalar(x, wl, fl, STOCHASTIC, SATURATE, 0) == hi
        assert R.fixed_scalar(x, wl, fl, STOCHASTIC, SATURATE, t) == lo
        assert R.fixed_scalar(x, wl, fl, STOCHASTIC, SATURATE, 0xFFFFFFFF) == lo


def test_stochastic_is_unbiased():
    """E[Q(x)] = x: the mean over many independent words is within 4 standard errors of x, and the
    frequency of rounding up follows the fraction f."""
    wl, fl, n = 12, 6, 1 << 16
    for x0 in (0.3, 0.01, -0.77, 1.0 / 3.0, 0.0001):
        x = np.full(n, x0, dtype=np.float32)
        q = R.fixed_quantize(x, wl, fl, STOCHASTIC, SATURATE, seed=4321, stream_id=5).astype(np.float64)
        step = 2.0 ** -fl
        assert set(np.unique(q)).issubset({np.floor(float(np.float32(x0)) / step) * step,
                                           np.ceil(float(np.float32(x0)) / step) * step})
        f = float(np.float32(x0)) / step - np.floor(float(np.float32(x0)) / step)
        sigma = step * np.sqrt(max(f * (1 - f), 1e-12) / n)
        assert abs(q.mean() - float(np.float32(x0))) < 4 * sigma + 1e-12
    # over seeds on a mixed tensor: the average of many quantizations converges to the input
    x = (W.normal_tensor(4096, seed=31) * np.float32(0.5)).astype(np.float32)
    acc = np.zeros(x.size)
    seeds = 256
    for s in range(seeds):
        acc += R.fixed_quantize(x, 12, 6, STOCHASTIC, SATURATE, seed=1000 + s)
    err = acc / seeds - x
    assert np.abs(err).max() < 5 * (2.0 ** -6) * 0.5 / np.sqrt(seeds)
    assert abs(err.mean()) < 4 * (2.0 ** -6) * 0.5 / np.sqrt(seeds * x.size)


@pytest.mark.parametrize("rounding", [RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC])
@pytest.mark.parametrize("flags", [0, SATURATE, SATURATE | SYMMETRIC])
def test_invariants(rounding, flags):
    wl, fl = 8, 6
    x = np.concatenate([W.uniform_with_outliers(30000, seed=2), W.mixed_scales(5000, seed=3, lo_exp=-30, hi_exp=20)])
    q = R.fixed_quantize(x, wl, fl, rounding, flags, seed=7)
    step = 2.0 ** -fl
    # members of the value set
    k = q.astype(np.float64) / step
    assert np.all(k == np.round(k))
    if flags & SATURATE:
        lo = -(2 ** (wl - 1)) + (1 if flags & SYMMETRIC else 0)
        assert k.min() >= lo and k.max() <= 2 ** (wl - 1) - 1
        inside = np.abs(x.astype(np.float64)) < (2 ** (wl - 1) - 1) * step
    else:
        inside = np.ones(x.size, dtype=bool)
    # error bound: half a step for nearest, less than one step for stochastic
    err = np.abs(q.astype(np.float64) - x.astype(np.float64))[inside]
    assert err.max() <= (step / 2 if rounding != STOCHASTIC else step * (1 - 1e-12))
    # idempotent, for any random word
    assert_bit_equal(R.fixed_quantize(q, wl, fl, rounding, flags, seed=99), q, "idempotence")
    # odd symmetry with the same random words (away from the asymmetric clamp)
    qn = R.fixed_quantize(-x, wl, fl, rounding, flags, seed=7)
    sym = inside if not (flags & SYMMETRIC) else np.ones(x.size, dtype=bool)
    assert_bit_equal(qn[sym], -q[sym], "odd symmetry")
    # sign of zero is kept
    z = R.fixed_quantize(np.array([0.0, -0.0, 1e-9, -1e-9], dtype=np.float32), wl, fl, RN_EVEN, flags)
    assert list(np.signbit(z)) == [False, True, False, True] and np.all(z == 0)


@pytest.mark.parametrize("rounding", [RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC])
def test_monotone_for_a_fixed_word(rounding):
    g = np.random.Generator(np.random.PCG64(5))
    xs = np.sort(np.concatenate([g.uniform(-2.5, 2.5, 3000), np.arange(-160, 160) / 128.0]).astype(np.float32))
    for r in (0, 0x40000000, 0x80000000, 0xFFFFFFFF, 123456789):
        q = np.array([R.fixed_scalar(x, 8, 6, rounding, SATURATE, r) for x in xs])
        assert np.all(np.diff(q) >= 0)


def test_nonfinite_and_validation():
    nan = np.array([np.nan], dtype=np.float32)
    nan.view(np.uint32)[0] = 0x7FC12345
    for flags in (0, SATURATE):
        assert R.fixed_quantize(nan, 8, 6, RN_EVEN, flags).view(np.uint32)[0] == 0x7FC12345
    inf = np.array([np.inf, -np.inf], dtype=np.float32)
    assert list(R.fixed_quantize(inf, 8, 6, RN_EVEN, SATURATE)) == [1.984375, -2.0]
    assert list(R.fixed_quantize(inf, 8, 6, RN_EVEN, 0)) == [np.inf, -np.inf]
    x = np.zeros(4, dtype=np.float32)
    for bad in [dict(wl=0, fl=0), dict(wl=25, fl=0), dict(wl=8, fl=150), dict(wl=8, fl=-121)]:
        with pytest.raises(R.OracleError) as e:
            R.fixed_quantize(x, bad["wl"], bad["fl"])
        assert e.value.status == 2
    with pytest.raises(R.OracleError) as e:
        R.fixed_quantize(x, 8, 6, rounding=4)
    assert e.value.status == 3
    with pytest.raises(R.OracleError) as e:
        R.fixed_quantize(x, 8, 6, flags=8)
    assert e.value.status == 2
    assert R.fixed_quantize(np.zeros(0, dtype=np.float32), 8, 6).size == 0


def test_threads_do_not_change_the_result():
    x = W.uniform_with_outliers(100003, seed=9)
    a = R.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=1234)
    b = R.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=1234, threads=7)
    assert_bit_equal(a, b, "thread split")


@pytest.mark.parametrize("index0", [0, 4, 7, (1 << 32) - 4, (1 << 32) - 1, 1 << 34])
def test_array_form_takes_the_word_of_the_elements_index(index0):
    """Sec. 3.1 "Rounding mode", stochastic: element i of an array that starts at element index0 of a
    tensor is rounded with random_word(seed, stream_id, role 0, index0 + i) — the scalar quantizer
    and the word generator are pinned on their own; this pins how the array form wires them."""
    seed, stream = 0xFEDCBA9876543210, 0x9E3779B9
    x = W.uniform_with_outliers(301, seed=31)
    got = R.fixed_quantize_at(x, index0, 8, 6, STOCHASTIC, SATURATE, seed=seed, stream_id=stream)
    want = np.array([R.fixed_scalar(x[i], 8, 6, STOCHASTIC, SATURATE, R.random_word(seed, stream, 0, index0 + i))
                     for i in range(x.size)], dtype=np.float32)
    assert_bit_equal(got, want, f"array form at index0 = {index0}")
    # the choice of word matters on this input: another role, stream, seed half or offset changes results
    for other in (R.random_words(seed, stream, 1, x.size, index0), R.random_words(seed, stream + 1, 0, x.size, index0),
                  R.random_words(seed >> 32, stream, 0, x.size, index0), R.random_words(seed, stream, 0, x.size, index0 + 1),
                  R.random_words(seed, stream, 0, x.size, 0 if index0 else 4)):
        alt = np.array([R.fixed_scalar(x[i], 8, 6, STOCHASTIC, SATURATE, int(other[i])) for i in range(x.size)],
                       dtype=np.float32)
        assert np.any(alt.view(np.uint32) != want.view(np.uint32))
    # the plain form is the array form at index0 = 0, split over threads or not
    if index0 == 0:
        assert_bit_equal(R.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=seed, stream_id=stream), want, "plain form")
        assert_bit_equal(R.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=seed, stream_id=stream, threads=5), want,
                         "plain form over threads")
