"""The size sweep of Sec. 4 "Validation" (fused kernels against the same quantization written as a
chain of stock tensor operations, over tensor sizes): both sides against the oracle, and the sweep
itself on a few small sizes."""
import numpy as np
import pytest

from oracle import qsim_ref as R
from paper_1910_04540_amd import workloads as W
from helpers import RN_EVEN, SATURATE, assert_bit_equal

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _tensor(log2n):
    base = W.normal_tensor(1 << 20, seed=21)
    n = 1 << log2n
    return np.ascontiguousarray(np.tile(base, (n + base.size - 1) // base.size)[:n])


@pytest.mark.parametrize("log2n", [10, 16, 22])
def test_fused_and_many_kernel_agree_with_the_oracle(log2n):
    from paper_1910_04540_amd import binding as Q
    from paper_1910_04540_amd import sweep

    x = _tensor(log2n)
    n = x.size
    d = torch.from_numpy(x).cuda()
    host = lambda t: t.cpu().numpy()

    # fixed point (8, 6), nearest even, saturating: the chain scales exactly, rounds half to even with
    # the library's round, clamps and scales back, which is the definition itself; signed zeros
    # included (a negative value that rounds to zero keeps its sign on both sides)
    want = R.fixed_quantize(x, 8, 6, RN_EVEN, SATURATE)
    assert_bit_equal(host(Q.fixed_quantize(d, 8, 6, Q.RN_EVEN, Q.SATURATE)), want, f"fused fixed 2^{log2n}")
    assert_bit_equal(host(sweep.many_fixed(d, 8, 6, False)), want, f"many-kernel fixed 2^{log2n}")

    # block floating point over the whole tensor.  The chain takes the shared exponent from
    # floor(log2(max |x|)) in fp32, which equals the exponent field unless the maximum lies within
    # rounding distance below a power of two; the maximum of these inputs does not (checked), so the
    # two definitions coincide here.  Where they would not, the fused kernel is the one that follows
    # the oracle (tests/test_gpu_parity.py covers maxima just below powers of two).
    amax = float(np.abs(x).max())
    assert amax > 0 and 1.0001 < amax / 2.0 ** np.floor(np.log2(amax)) < 1.9999
    want = R.block_quantize(x, 1, 1, n, 8, RN_EVEN)
    assert_bit_equal(host(Q.block_quantize(d, 1, 1, n, 8, Q.RN_EVEN)), want, f"fused block 2^{log2n}")
    assert_bit_equal(host(sweep.many_block(d, 8, False)), want, f"many-kernel block 2^{log2n}")

    # the stochastic chains draw their own random numbers, so only their value sets can be compared:
    # every result is on the format's grid and within one step of the input
    for got in (host(sweep.many_fixed(d, 8, 6, True)), host(Q.fixed_quantize(d, 8, 6, Q.STOCHASTIC, Q.SATURATE, seed=3))):
        k = got.astype(np.float64) * 64.0
        assert np.array_equal(k, np.rint(k)) and k.min() >= -128 and k.max() <= 127
        inside = np.abs(x) < 1.9
        assert np.all(np.abs(got[inside].astype(np.float64) - x[inside]) < 1.0 / 64.0)


def test_the_sweep_runs_and_prints_its_rows():
    from paper_1910_04540_amd import sweep

    rows = sweep.size_sweep(10, 14, step=2, reps=3)
    assert [(r["log2_n"], r["rounding"]) for r in rows] == [(10, "nearest"), (10, "stochastic"), (12, "nearest"),
                                                             (12, "stochastic"), (14, "nearest"), (14, "stochastic")]
    for r in rows:
        for key in ("fixed_fused_us", "fixed_many_us", "block_fused_us", "block_many_us", "float_fused_us"):
            assert r[key] > 0.0
    text = sweep.format_rows(rows)
    assert text.count("\n") == len(rows) and "2^12" in text and "stochastic" in text
