"""Host-side logic of the front-end descriptors (no GPU needed)."""
import pytest

torch = pytest.importorskip("torch")
from paper_1910_04540_amd import quantizer as Z     # noqa: E402


def test_block_layouts():
    shape = (6, 5, 7)
    assert Z.BlockFloatingPoint(8, None).layout(shape) == (1, 1, 210)
    assert Z.BlockFloatingPoint(8, 0).layout(shape) == (1, 6, 35)
    assert Z.BlockFloatingPoint(8, 1).layout(shape) == (6, 5, 7)
    assert Z.BlockFloatingPoint(8, 2).layout(shape) == (30, 7, 1)
    assert Z.BlockFloatingPoint(8, -1).layout(shape) == (30, 7, 1)
    assert Z.BlockFloatingPoint(8, 0).layout((9,)) == (1, 9, 1)


def test_flags_and_rounding_names():
    assert Z.FloatingPoint(5, 2).flags() == 1 and Z.FloatingPoint(5, 2, subnormal=True).flags() == 3
    assert Z.FloatingPoint(8, 7, saturate=False).flags() == 0
    assert Z.FixedPoint(8, 6).flags() == 1 and Z.FixedPoint(8, 6, clamp=False, symmetric=True).flags() == 4
    assert Z.BlockFloatingPoint(8).flags() == 0 and Z.BlockFloatingPoint(8, symmetric=True).flags() == 4
    assert [Z._rounding(k) for k in ("nearest", "nearest_away", "nearest_zero", "stochastic")] == [0, 1, 2, 3]
    with pytest.raises(ValueError):
        Z._rounding("banker")
    q = Z.Quantizer(Z.FixedPoint(8, 6), None, "stochastic", "nearest", seed=4)
    assert (q.forward_rounding, q.backward_rounding, q.seed, q.calls) == (3, 0, 4, 0)
    assert "FixedPoint" in repr(q)


def test_formats_of_the_sgd_step():
    from paper_1910_04540_amd import binding as B
    from paper_1910_04540_amd.optim import sgd_format

    def fields(f):
        return (f.kind, f.a, f.b, f.rounding, f.flags)

    assert fields(sgd_format(None)) == (B.KIND_IDENTITY, 0, 0, 0, 0)
    assert fields(sgd_format(Z.FloatingPoint(5, 2, subnormal=True), "stochastic")) == (B.KIND_FLOAT, 5, 2, 3, 3)
    assert fields(sgd_format(Z.FixedPoint(16, 12), "nearest_away")) == (B.KIND_FIXED, 16, 12, 1, 1)
    assert fields(sgd_format(Z.BlockFloatingPoint(8, symmetric=True), "nearest", chunk=128)) == (B.KIND_BLOCK, 8, 128, 0, 4)
    with pytest.raises(ValueError):
        sgd_format(Z.BlockFloatingPoint(8, dim=0))
    with pytest.raises(TypeError):
        sgd_format("fp16")


def test_modules_without_a_seed_do_not_share_random_words():
    a, b = Z.Quantizer(Z.FixedPoint(8, 6)), Z.Quantizer(Z.FixedPoint(8, 6))
    assert a.seed != b.seed and a.seed >= 1 << 32 and b.seed >= 1 << 32
    assert Z.Quantizer(Z.FixedPoint(8, 6), seed=7).seed == 7
