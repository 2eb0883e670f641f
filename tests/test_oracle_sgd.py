"""Pins for the oracle's quantized SGD-with-momentum step (Sec. 3.1 "Front-end interface";
Sec. 1 footnote 1 for the fp32 master copy)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qsim_ref as R
from paper_1910_04540_amd import workloads as W
from helpers import (RN_EVEN, STOCHASTIC, SATURATE, SUBNORMAL, assert_bit_equal, f32_to_fraction,
                     round_fraction_to_f32)

IDENT = R.Format(0, 0, 0, 0, 0)


def test_identity_formats_give_textbook_sgd_with_one_rounding_per_fma():
    """With every format the identity the step is v' = fl(mu*v + g), w' = fl(w - lr*v'), each a
    single correctly rounded operation: checked in exact rational arithmetic."""
    n = 400
    w, g, m = W.sgd_state(n)
    lr, mu = np.float32(0.1), np.float32(0.9)
    w2, wq, m2 = R.quant_sgd_step(w, g, m, lr, mu, IDENT, IDENT, IDENT)
    for i in range(n):
        v = round_fraction_to_f32(f32_to_fraction(mu) * f32_to_fraction(m[i]) + f32_to_fraction(g[i]))
        assert m2[i] == v
        wi = round_fraction_to_f32(f32_to_fraction(w[i]) - f32_to_fraction(lr) * f32_to_fraction(v))
        assert w2[i] == wi
    assert_bit_equal(wq, w2, "identity weight format copies the master weights")
    # a product that is not representable shows a fused operation differs from two roundings
    a = np.float32(1.0 + 2.0 ** -12)
    two_step = np.float32(np.float32(a * a) + np.float32(-1.0))
    one_step = round_fraction_to_f32(f32_to_fraction(a) ** 2 - 1)
    assert two_step != one_step
    w2, _, m2 = R.quant_sgd_step(np.zeros(1, np.float32), np.array([-1.0], np.float32), np.array([a], np.float32),
                                 0.0, a, IDENT, IDENT, IDENT)
    assert m2[0] == one_step


@pytest.mark.parametrize("fg,fm,fw", [
    (R.Format(1, 5, 2, STOCHASTIC, SATURATE | SUBNORMAL), R.Format(2, 16, 12, STOCHASTIC, SATURATE), R.Format(3, 8, 256, RN_EVEN, 0)),
    (R.Format(2, 8, 10, RN_EVEN, SATURATE), R.Format(1, 8, 7, RN_EVEN, SATURATE), R.Format(1, 5, 10, STOCHASTIC, SATURATE | SUBNORMAL)),
    (R.Format(3, 8, 64, STOCHASTIC, 0), R.Format(3, 12, 1024, STOCHASTIC, 0), R.Format(3, 6, 4, STOCHASTIC, 0)),
    (IDENT, R.Format(2, 16, 12, STOCHASTIC, SATURATE), R.Format(2, 8, 6, STOCHASTIC, SATURATE)),
])
@pytest.mark.parametrize("n", [2048, 1000])
def test_step_is_the_composition_of_the_pinned_quantizers(fg, fm, fw, n):
    """The step equals: quantize the gradient array, one fma, quantize, one fma, quantize, built
    from the array quantizers pinned elsewhere.  Random words: role 0/1/2, same seed and stream."""
    w, g, m = W.sgd_state(n)
    lr, mu, seed, stream = np.float32(0.1), np.float32(0.9), 1234, 3

    def q(x, f, role):
        if f.kind == 0:
            return x.copy()
        words = None
        if f.rounding == STOCHASTIC:
            words = R.random_words(seed, stream, role, x.size)
        out = np.empty_like(x)
        if f.kind == 3:
            for c0 in range(0, x.size, f.b):
                blk = x[c0:c0 + f.b]
                e_s = int(R.block_exponents(blk, 1, 1, blk.size)[0])
                for i, v in enumerate(blk):
                    out[c0 + i] = R.fixed_scalar(v, f.a, f.a - 2 - e_s, f.rounding, SATURATE | (f.flags & 4),
                                                 int(words[c0 + i]) if words is not None else 0)
            return out
        fn = R.float_scalar if f.kind == 1 else R.fixed_scalar
        for i, v in enumerate(x):
            out[i] = fn(v, f.a, f.b, f.rounding, f.flags, int(words[i]) if words is not None else 0)
        return out

    def fma(a, b, c):
        return np.array([round_fraction_to_f32(f32_to_fraction(a) * f32_to_fraction(bi) + f32_to_fraction(ci))
                         for bi, ci in zip(b, c)], dtype=np.float32)

    gq = q(g, fg, 0)
    v = q(fma(mu, m, gq), fm, 1)
    wn = fma(-lr, v, w)
    wq_want = q(wn, fw, 2)
    w2, wq, m2 = R.quant_sgd_step(w, g, m, lr, mu, fg, fm, fw, seed, stream)
    assert_bit_equal(m2, v, "momentum")
    assert_bit_equal(w2, wn, "master weights")
    assert_bit_equal(wq, wq_want, "quantized weights")
    w3, none, m3 = R.quant_sgd_step(w, g, m, lr, mu, fg, fm, fw, seed, stream, want_wq=False)
    assert none is None
    assert_bit_equal(w3, w2, "w without w_q") and assert_bit_equal(m3, m2, "mom without w_q")


def test_weights_kept_in_the_weight_format():
    """w_q = w_master: the stored weights are Qw of the fp32 update, and the next step starts from them."""
    w, g, m = W.sgd_state(777)
    fg, fm, fw = R.Format(1, 5, 2, STOCHASTIC, SATURATE | SUBNORMAL), R.Format(2, 16, 12, STOCHASTIC, SATURATE), R.Format(3, 8, 64, RN_EVEN, 0)
    w1, wq1, m1 = R.quant_sgd_step(w, g, m, 0.1, 0.9, fg, fm, fw, 5, 2)
    a1, aq1, am1 = R.quant_sgd_step(w, g, m, 0.1, 0.9, fg, fm, fw, 5, 2, in_place_weights=True)
    assert_bit_equal(a1, wq1, "stored weights are the quantized ones")
    assert_bit_equal(am1, m1, "momentum unaffected")
    assert aq1 is a1
    a2, _, _ = R.quant_sgd_step(a1, g, am1, 0.1, 0.9, fg, fm, fw, 5, 3, in_place_weights=True)
    w2, wq2, _ = R.quant_sgd_step(wq1, g, m1, 0.1, 0.9, fg, fm, fw, 5, 3)
    assert_bit_equal(a2, wq2, "second step from quantized weights")


@pytest.mark.parametrize("wd,damp,nesterov", [(5e-4, 0.0, 0), (0.0, 0.25, 0), (0.0, 0.0, 1), (5e-4, 0.0, 1), (1e-2, 0.5, 0)])
def test_options_one_correctly_rounded_operation_per_line(wd, damp, nesterov):
    """Weight decay, dampening and Nesterov momentum with identity formats, each line of the header
    checked as a single correctly rounded fp32 operation in exact rational arithmetic."""
    n = 300
    w, g, m = W.sgd_state(n)
    lr, mu = np.float32(0.1), np.float32(0.9)
    F = f32_to_fraction
    opt = R.SgdOptions(wd, damp, nesterov)
    w2, _, m2 = R.quant_sgd_step(w, g, m, lr, mu, IDENT, IDENT, IDENT, options=opt)
    wd32, keep = np.float32(wd), np.float32(np.float32(1.0) - np.float32(damp))
    for i in range(n):
        d = round_fraction_to_f32(F(wd32) * F(w[i]) + F(g[i])) if wd else g[i]
        t = round_fraction_to_f32(F(keep) * F(d)) if damp else d
        v = round_fraction_to_f32(F(mu) * F(m[i]) + F(t))
        step = round_fraction_to_f32(F(mu) * F(v) + F(d)) if nesterov else v
        wn = round_fraction_to_f32(F(w[i]) - F(lr) * F(step))
        assert m2[i] == v and w2[i] == wn, (i, m2[i], v, w2[i], wn)


@pytest.mark.parametrize("wd,damp,nesterov", [(0.0, 0.0, False), (5e-4, 0.0, False), (5e-4, 0.0, True), (1e-3, 0.3, False)])
def test_options_follow_pytorch_sgd(wd, damp, nesterov):
    """Five steps with identity formats track torch.optim.SGD (an independent implementation of the
    same update rule) to within a few roundings: pins the order of the terms and their signs."""
    torch = pytest.importorskip("torch")
    n = 2000
    w, _, _ = W.sgd_state(n)
    p = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.SGD([p], lr=0.05, momentum=0.9, weight_decay=wd, dampening=damp, nesterov=nesterov)
    wr, mr = w.copy(), np.zeros(n, dtype=np.float32)
    for step in range(5):
        g = W.sgd_state(n, seeds=(50 + step, 60 + step, 70 + step))[1] * np.float32(30.0)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        if step == 0 and damp:
            # PyTorch seeds the momentum buffer with the undamped gradient on its first step
            mr = (g + np.float32(wd) * wr).astype(np.float32) if wd else g.copy()
            wr = (wr - np.float32(0.05) * mr).astype(np.float32)
            continue
        wr, _, mr = R.quant_sgd_step(wr, g, mr, 0.05, 0.9, IDENT, IDENT, IDENT, options=R.SgdOptions(wd, damp, int(nesterov)),
                                     want_wq=False)
    np.testing.assert_allclose(wr, p.detach().numpy(), rtol=2e-5, atol=1e-7)
    assert np.abs(wr - w).max() > 1e-3          # the weights did move


def test_options_with_quantizers_compose():
    """With formats, the options sit between the pinned quantizers exactly as the header says."""
    n = 1500
    w, g, m = W.sgd_state(n)
    fg, fm, fw = R.Format(1, 5, 2, STOCHASTIC, SATURATE | SUBNORMAL), R.Format(2, 16, 12, STOCHASTIC, SATURATE), R.Format(3, 8, 256, RN_EVEN, 0)
    lr, mu, wd, damp = np.float32(0.1), np.float32(0.9), np.float32(5e-4), np.float32(0.125)
    F = f32_to_fraction
    fma = lambda a, b, c: np.array([round_fraction_to_f32(F(a) * F(x) + F(y)) for x, y in zip(b, c)], dtype=np.float32)
    gq = R.float_quantize(g, 5, 2, STOCHASTIC, SATURATE | SUBNORMAL, 9, 4)
    d = fma(wd, w, gq)
    t = (np.float32(np.float32(1) - damp) * d).astype(np.float32)
    w2, wq, m2 = R.quant_sgd_step(w, g, m, lr, mu, fg, fm, fw, 9, 4, options=R.SgdOptions(wd, damp, 1))
    words = R.random_words(9, 4, 1, n)
    v = np.array([R.fixed_scalar(x, 16, 12, STOCHASTIC, SATURATE, int(r)) for x, r in zip(fma(mu, m, t), words)], dtype=np.float32)
    assert_bit_equal(m2, v, "momentum")
    wn = fma(-lr, fma(mu, v, d), w)
    assert_bit_equal(w2, wn, "weights (Nesterov)")
    assert_bit_equal(wq, R.block_quantize(wn, 1, (n + 255) // 256, 256, 8, RN_EVEN), "quantized weights")


def test_validation():
    w, g, m = W.sgd_state(64)
    bad = [R.Format(4, 0, 0, 0, 0), R.Format(1, 9, 2, 0, 0), R.Format(2, 30, 2, 0, 0), R.Format(3, 8, 100, 0, 0),
           R.Format(3, 8, 2048, 0, 0), R.Format(3, 1, 64, 0, 0), R.Format(2, 8, 6, 0, 16)]
    for f in bad:
        with pytest.raises(R.OracleError) as e:
            R.quant_sgd_step(w, g, m, 0.1, 0.9, f, IDENT, IDENT)
        assert e.value.status == 2
    with pytest.raises(R.OracleError) as e:
        R.quant_sgd_step(w, g, m, 0.1, 0.9, IDENT, R.Format(2, 8, 6, 7, 0), IDENT)
    assert e.value.status == 3
