"""Pins for the oracle's custom floating point (Sec. 3.1 "Number Formats", first paragraph)."""
import os

import numpy as np
import pytest

from oracle import qsim_ref as R
from paper_1910_04540_amd import workloads as W
from helpers import (RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC, SATURATE, SUBNORMAL, model_float,
                     assert_bit_equal)

torch = pytest.importorskip("torch")


def test_spot_values(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "spot_values.txt")) as fh:
        rows = [line.split()[1:] for line in fh if line.startswith("float ")]
    assert len(rows) >= 15
    for e, m, rounding, flags, x, want in rows:
        got = R.float_scalar(float(x), int(e), int(m), int(rounding), int(flags))
        assert float(got) == float(want), (e, m, rounding, flags, x, got, want)


def _probe(dropped_bits):
    x = W.all_exponents_probe(dropped_bits)
    return x[np.isfinite(x)]


def test_e5m10_is_binary16_conversion():
    """(5, 10), nearest-even, gradual underflow == IEEE binary16 conversion (numpy's float16),
    over every exponent and every class of dropped bits, below the overflow threshold 65520."""
    x = _probe(13)
    x = x[np.abs(x) < 65520.0]
    got = R.float_quantize(x, 5, 10, RN_EVEN, SATURATE | SUBNORMAL, threads=8)
    assert_bit_equal(got, x.astype(np.float16).astype(np.float32), "E5M10 vs float16")
    # the sub-range where binary16 is subnormal needs every low-bit pattern to matter: dense sweep
    dense = np.arange(0x33000000, 0x38800000, 37, dtype=np.uint32).view(np.float32)   # 2^-25 .. 2^-14
    got = R.float_quantize(dense, 5, 10, RN_EVEN, SATURATE | SUBNORMAL, threads=8)
    assert_bit_equal(got, dense.astype(np.float16).astype(np.float32), "E5M10 subnormal range")
    # unsaturated, the oracle keeps growing where binary16 overflows
    assert R.float_scalar(70000.0, 5, 10, RN_EVEN, SUBNORMAL) == 70016.0


def test_e8m7_is_bfloat16_conversion():
    x = _probe(16)
    x = x[np.abs(x) < 3.38e38]
    got = R.float_quantize(x, 8, 7, RN_EVEN, SATURATE | SUBNORMAL, threads=8)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert_bit_equal(got, want, "E8M7 vs bfloat16")


def test_e5m2_is_float8_e5m2_conversion():
    if not hasattr(torch, "float8_e5m2"):
        pytest.skip("installed torch has no float8_e5m2")
    x = _probe(21)
    x = x[np.abs(x) < 61440.0]
    got = R.float_quantize(x, 5, 2, RN_EVEN, SATURATE | SUBNORMAL, threads=8)
    want = torch.from_numpy(x).to(torch.float8_e5m2).to(torch.float32).numpy()
    assert_bit_equal(got, want, "E5M2 vs float8_e5m2")


def test_e8m23_is_identity():
    x = np.concatenate([W.mixed_scales(20000, seed=5), np.array([0.0, -0.0, 1e-45, -1e-40], dtype=np.float32)])
    x = x[np.isfinite(x)]
    for rounding in (RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC):
        assert_bit_equal(R.float_quantize(x, 8, 23, rounding, SATURATE | SUBNORMAL, seed=3), x, "identity")


@pytest.mark.skipif(os.environ.get("QSIM_EXHAUSTIVE") != "1", reason="all 2^32 inputs: set QSIM_EXHAUSTIVE=1")
def test_e5m10_exhaustive_all_fp32():
    for start in range(0, 1 << 32, 1 << 26):
        x = np.arange(start, start + (1 << 26), dtype=np.uint64).astype(np.uint32).view(np.float32)
        keep = np.isfinite(x) & (np.abs(x) < 65520.0)
        got = R.float_quantize(x[keep], 5, 10, RN_EVEN, SATURATE | SUBNORMAL, threads=8)
        assert_bit_equal(got, x[keep].astype(np.float16).astype(np.float32), f"chunk {start:#x}")


@pytest.mark.parametrize("e,m", [(2, 1), (3, 2), (4, 3), (5, 2), (8, 2), (4, 1)])
@pytest.mark.parametrize("flags", [0, SATURATE, SUBNORMAL, SATURATE | SUBNORMAL])
def test_tiny_formats_by_value_set(e, m, flags):
    """Every mode against the explicitly enumerated value set, exact rational arithmetic."""
    g = np.random.Generator(np.random.PCG64(41))
    bias = (1 << (e - 1)) - 1
    lo, hi = (1 - bias) - m - 4, bias + 3
    xs = np.concatenate([
        W.mixed_scales(400, seed=42, lo_exp=lo, hi_exp=hi),
        # midpoints between neighbouring values of a few binades, and their fp32 neighbours
        np.array([(1 + (2 * j + 1) / 2 ** (m + 1)) * 2.0 ** b for j in range(1 << m) for b in (lo + 3, 1 - bias - 1, 1 - bias, 0, bias)],
                 dtype=np.float32),
        np.array([(j + 0.5) / 2 ** m * 2.0 ** (1 - bias) for j in range(1 << m)], dtype=np.float32),
        np.array([0.0, -0.0, np.inf, -np.inf, 1e-45, -1e-45, 1.1754942e-38, 5.877472e-39, 3.4028235e38], dtype=np.float32),
    ])
    xs = np.concatenate([xs, np.nextafter(xs, np.float32(np.inf)), np.nextafter(xs, np.float32(-np.inf))])
    rs = g.integers(0, 1 << 32, size=xs.size, dtype=np.uint64)
    for rounding in (RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC):
        for x, r in zip(xs, rs):
            got = R.float_scalar(x, e, m, rounding, flags, int(r))
            want = model_float(x, e, m, rounding, flags, int(r))
            assert got.view(np.uint32) == want.view(np.uint32), (x, hex(x.view(np.uint32)), rounding, flags, r, got, want)


def test_denormal_input_that_rounds_up_to_the_smallest_normal():
    """E = 8 without gradual underflow: an fp32 denormal is rounded with its true exponent, so the
    largest denormal rounds up to 2^-126 and survives the flush; smaller ones are flushed."""
    big = np.array([0x007FFFFF], dtype=np.uint32).view(np.float32)[0]
    assert R.float_scalar(big, 8, 7, RN_EVEN, SATURATE).view(np.uint32) == 0x00800000
    assert R.float_scalar(-big, 8, 7, RN_EVEN, SATURATE).view(np.uint32) == 0x80800000
    mid = np.array([0x00400000], dtype=np.uint32).view(np.float32)[0]
    assert R.float_scalar(mid, 8, 7, RN_EVEN, SATURATE).view(np.uint32) == 0x00000000
    assert R.float_scalar(mid, 8, 7, RN_EVEN, SATURATE | SUBNORMAL).view(np.uint32) == 0x00400000


@pytest.mark.parametrize("e,m", [(5, 2), (5, 10), (8, 7), (4, 3), (6, 9)])
@pytest.mark.parametrize("rounding", [RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC])
@pytest.mark.parametrize("flags", [0, SATURATE | SUBNORMAL, SATURATE])
def test_invariants(e, m, rounding, flags):
    bias = (1 << (e - 1)) - 1
    x = np.concatenate([W.normal_tensor(20000, seed=1),
                        W.mixed_scales(20000, seed=6, lo_exp=-bias - m - 5, hi_exp=min(bias + 4, 127))])
    q = R.float_quantize(x, e, m, rounding, flags, seed=17)
    # members of the value set: at most m mantissa bits, exponent within range
    nz = q != 0
    mant, ex = np.frexp(q[nz].astype(np.float64))            # q = mant * 2^ex, mant in [0.5, 1)
    ex = ex - 1
    if flags & SUBNORMAL:
        grid = np.exp2(np.maximum(ex, 1 - bias) - m)
    else:
        grid = np.exp2(ex - m)
        assert ex.min() >= 1 - bias
    kk = np.abs(q[nz].astype(np.float64)) / grid
    assert np.all(kk == np.round(kk))
    maxval = (2 - 2.0 ** -m) * 2.0 ** bias
    if flags & SATURATE:
        assert np.abs(q).max() <= maxval
    # idempotent
    assert_bit_equal(R.float_quantize(q, e, m, rounding, flags, seed=5), q, "idempotence")
    # odd symmetry
    assert_bit_equal(R.float_quantize(-x, e, m, rounding, flags, seed=17), -q, "odd symmetry")
    # relative error bound inside the normal range
    a = np.abs(x.astype(np.float64))
    inside = (a >= 2.0 ** (1 - bias)) & (a <= maxval)
    rel = np.abs(q.astype(np.float64) - x.astype(np.float64))[inside] / a[inside]
    assert rel.max() <= (2.0 ** -(m + 1) if rounding != STOCHASTIC else 2.0 ** -m)
    # sign of zero and of flushed values
    z = R.float_quantize(np.array([0.0, -0.0, 1e-44, -1e-44], dtype=np.float32), e, m, RN_EVEN, flags & ~SUBNORMAL)
    assert list(np.signbit(z)) == [False, True, False, True]


@pytest.mark.parametrize("rounding", [RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC])
@pytest.mark.parametrize("flags", [0, SATURATE | SUBNORMAL, SATURATE])
def test_monotone_for_a_fixed_word(rounding, flags):
    xs = np.sort(np.concatenate([W.mixed_scales(3000, seed=8, lo_exp=-22, hi_exp=18),
                                 W.normal_tensor(1000, seed=2)]))
    for r in (0, 0x80000000, 0xFFFFFFFF, 987654321):
        q = np.array([R.float_scalar(x, 5, 2, rounding, flags, r) for x in xs])
        assert np.all(np.diff(q) >= 0)


def test_stochastic_is_unbiased():
    n = 1 << 16
    for x0 in (1.1, 0.3, -3.3e-6, 40000.0):
        x = np.full(n, x0, dtype=np.float32)
        q = R.float_quantize(x, 5, 2, STOCHASTIC, SATURATE | SUBNORMAL, seed=77).astype(np.float64)
        vals = np.unique(q)
        assert 1 <= vals.size <= 2
        step = (vals.max() - vals.min()) if vals.size == 2 else 0.0
        assert abs(q.mean() - float(np.float32(x0))) <= 4 * step * 0.5 / np.sqrt(n) + 1e-30


def test_nonfinite_and_validation():
    nan = np.array([0x7FC00001, 0xFFC54321], dtype=np.uint32).view(np.float32)
    for flags in (0, SATURATE, SATURATE | SUBNORMAL):
        assert_bit_equal(R.float_quantize(nan, 5, 2, RN_EVEN, flags), nan, "NaN passes")
    inf = np.array([np.inf, -np.inf], dtype=np.float32)
    assert list(R.float_quantize(inf, 5, 2, RN_EVEN, SATURATE)) == [57344.0, -57344.0]
    assert list(R.float_quantize(inf, 5, 2, RN_EVEN, 0)) == [np.inf, -np.inf]
    # no saturation: only the carrier's own range ends the exponent
    assert R.float_scalar(3.4028235e38, 8, 7, RN_EVEN, 0) == np.inf
    assert R.float_scalar(3.4028235e38, 8, 7, RN_EVEN, SATURATE) == np.float32(3.3895314e38)
    x = np.zeros(4, dtype=np.float32)
    for e, m in [(1, 3), (9, 3), (5, 0), (5, 24)]:
        with pytest.raises(R.OracleError) as err:
            R.float_quantize(x, e, m)
        assert err.value.status == 2
    with pytest.raises(R.OracleError) as err:
        R.float_quantize(x, 5, 2, rounding=-1)
    assert err.value.status == 3


@pytest.mark.parametrize("index0", [0, 4, 7, (1 << 32) - 4, (1 << 32) - 1, 1 << 34])
@pytest.mark.parametrize("e,m,flags", [(5, 2, SATURATE | SUBNORMAL), (8, 7, 0)])
def test_array_form_takes_the_word_of_the_elements_index(index0, e, m, flags):
    """Sec. 3.1 "Rounding mode", stochastic: element i of an array that starts at element index0 of a
    tensor is rounded with random_word(seed, stream_id, role 0, index0 + i); pins how the array form
    wires the (separately pinned) scalar quantizer and word generator together."""
    seed, stream = 0xFEDCBA9876543210, 0x9E3779B9
    x = W.mixed_scales(301, seed=32)
    x = x[np.isfinite(x)]
    got = R.float_quantize_at(x, index0, e, m, STOCHASTIC, flags, seed=seed, stream_id=stream)
    want = np.array([R.float_scalar(x[i], e, m, STOCHASTIC, flags, R.random_word(seed, stream, 0, index0 + i))
                     for i in range(x.size)], dtype=np.float32)
    assert_bit_equal(got, want, f"array form at index0 = {index0}")
    for other in (R.random_words(seed, stream, 1, x.size, index0), R.random_words(seed, stream + 1, 0, x.size, index0),
                  R.random_words(seed >> 32, stream, 0, x.size, index0), R.random_words(seed, stream, 0, x.size, index0 + 1),
                  R.random_words(seed, stream, 0, x.size, 0 if index0 else 4)):
        alt = np.array([R.float_scalar(x[i], e, m, STOCHASTIC, flags, int(other[i])) for i in range(x.size)],
                       dtype=np.float32)
        assert np.any(alt.view(np.uint32) != want.view(np.uint32))
    if index0 == 0:
        assert_bit_equal(R.float_quantize(x, e, m, STOCHASTIC, flags, seed=seed, stream_id=stream), want, "plain form")
        assert_bit_equal(R.float_quantize(x, e, m, STOCHASTIC, flags, seed=seed, stream_id=stream, threads=5), want,
                         "plain form over threads")
