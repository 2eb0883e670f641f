"""Seeded random block shapes: every kernel form the dispatcher can pick (teams, whole workgroups,
ragged rows, single pass, block by block, flat, column, two-pass), with random word lengths,
rounding modes, flags, alignment offsets, in place or not, against the oracle bit for bit."""
import numpy as np
import pytest

from helpers import assert_bit_equal

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import qsim_ref as R                          # noqa: E402
from paper_1910_04540_amd import binding as Q             # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")


def _log_uniform(g, lo, hi):
    return int(round(float(np.exp(g.uniform(np.log(lo), np.log(hi))))))


def _shape(g, cap):
    """(outer, nblocks, inner) with at most `cap` elements, spread over orders of magnitude."""
    while True:
        kind = g.integers(0, 4)
        if kind == 0:                                   # contiguous blocks
            outer, nblocks, inner = 1, _log_uniform(g, 1, 20000), _log_uniform(g, 1, 200000)
        elif kind == 1:                                 # whole tensor
            outer, nblocks, inner = 1, 1, _log_uniform(g, 1, cap)
        else:                                           # blocks along an inner dimension
            outer, nblocks, inner = _log_uniform(g, 2, 5000), _log_uniform(g, 1, 5000), _log_uniform(g, 1, 70000)
        if g.integers(0, 3) == 0:
            inner = max(4, inner // 4 * 4)              # whole groups, often
        if outer * nblocks * inner <= cap:
            return outer, nblocks, inner


@pytest.mark.parametrize("seed", range(40))
def test_random_block_shapes(seed):
    g = np.random.Generator(np.random.PCG64(1000 + seed))
    for case in range(25):
        outer, nblocks, inner = _shape(g, 6_000_000 if case % 5 == 0 else 1_000_000)
        n = outer * nblocks * inner
        if outer == 1 and nblocks > 1 and g.integers(0, 3) == 0:
            n -= int(g.integers(0, inner))              # a short last block
        wl = int(g.integers(2, 25))
        rounding = int(g.integers(0, 4))
        flags = int(g.choice([0, R.SYMMETRIC]))
        offset = int(g.choice([0, 0, 1, 2, 3]))
        in_place = bool(g.integers(0, 2))
        scale = np.exp2(g.integers(-30, 30, size=nblocks)).astype(np.float32)
        if outer == 1:
            x = g.standard_normal(nblocks * inner, dtype=np.float32).reshape(nblocks, inner) * scale[:, None]
            x = x.reshape(-1)[:n].astype(np.float32)
        else:
            x = (g.standard_normal((outer, nblocks, inner), dtype=np.float32) * scale[None, :, None]).astype(np.float32).reshape(-1)
        if n > 3 and g.integers(0, 4) == 0:
            x[int(g.integers(0, n))] = np.float32(g.choice([np.inf, -np.inf, np.nan, 3.0e38, 0.0]))
        seed64, stream = int(g.integers(0, 2 ** 62)), int(g.integers(0, 2 ** 32))
        want = R.block_quantize(x, outer, nblocks, inner, wl, rounding, flags, seed64, stream)
        what = f"seed {seed} case {case}: [{outer},{nblocks},{inner}] n={n} wl={wl} mode={rounding} flags={flags} offset={offset} in_place={in_place}"
        pad = torch.from_numpy(np.concatenate([np.zeros(offset, np.float32), x, np.zeros(5, np.float32)])).cuda()
        view = pad[offset:offset + n]
        out = view if in_place else torch.empty(n + 1, device="cuda")[1 - (offset & 1):][:n]
        Q.block_quantize(view, outer, nblocks, inner, wl, rounding, flags, seed64, stream, out=out)
        torch.cuda.synchronize()
        assert_bit_equal(out.cpu().numpy(), want, what)
        full = pad.cpu().numpy()
        assert not full[:offset].any() and not full[offset + n:].any(), what + ": wrote outside the array"


@pytest.mark.parametrize("seed", range(4))
def test_random_elementwise_and_sgd(seed):
    g = np.random.Generator(np.random.PCG64(5000 + seed))
    for case in range(20):
        n = _log_uniform(g, 1, 2_000_000)
        offset = int(g.choice([0, 1, 2, 3]))
        x = (g.standard_normal(n, dtype=np.float32) * np.exp2(g.integers(-40, 40, size=n))).astype(np.float32)
        rounding = int(g.integers(0, 4))
        seed64, stream = int(g.integers(0, 2 ** 62)), int(g.integers(0, 2 ** 32))
        d = torch.from_numpy(np.concatenate([np.zeros(offset, np.float32), x])).cuda()[offset:]
        e, m = int(g.integers(2, 9)), int(g.integers(1, 24))
        fl_flags = int(g.integers(0, 4))
        assert_bit_equal(Q.float_quantize(d, e, m, rounding, fl_flags, seed64, stream).cpu().numpy(),
                         R.float_quantize(x, e, m, rounding, fl_flags, seed64, stream),
                         f"seed {seed} case {case}: float({e},{m}) n={n} mode={rounding} flags={fl_flags} offset={offset}")
        wl = int(g.integers(1, 25))
        fl = int(g.integers(wl - 40, 60))
        fx_flags = int(g.choice([0, 1, 1 | 4, 4]))
        assert_bit_equal(Q.fixed_quantize(d, wl, fl, rounding, fx_flags, seed64, stream).cpu().numpy(),
                         R.fixed_quantize(x, wl, fl, rounding, fx_flags, seed64, stream),
                         f"seed {seed} case {case}: fixed({wl},{fl}) n={n} mode={rounding} flags={fx_flags} offset={offset}")


def _random_format(g):
    kind = int(g.integers(0, 4))
    rounding = int(g.integers(0, 4))
    if kind == 0:
        return (0, 0, 0, 0, 0)
    if kind == 1:
        return (1, int(g.integers(2, 9)), int(g.integers(1, 24)), rounding, int(g.integers(0, 4)))
    if kind == 2:
        wl = int(g.integers(1, 25))
        return (2, wl, int(g.integers(wl - 20, 40)), rounding, int(g.choice([0, 1, 5, 4])))
    return (3, int(g.integers(2, 25)), int(2 ** g.integers(2, 11)), rounding, int(g.choice([0, 4])))


@pytest.mark.parametrize("seed", range(6))
def test_random_sgd_steps(seed):
    g = np.random.Generator(np.random.PCG64(9000 + seed))
    for case in range(15):
        n = _log_uniform(g, 1, 1_000_000)
        offset = int(g.choice([0, 0, 1, 3]))
        fmts = [_random_format(g) for _ in range(3)]
        opts = (float(g.choice([0.0, 5e-4])), float(g.choice([0.0, 0.25])), int(g.integers(0, 2)))
        mode = str(g.choice(["copy", "in_place", "none"]))
        lr, mu = float(g.choice([0.1, 0.01])), float(g.choice([0.0, 0.9]))
        w = (g.standard_normal(n, dtype=np.float32) * np.float32(0.05)).astype(np.float32)
        gr = (g.standard_normal(n, dtype=np.float32) * np.exp2(g.integers(-20, 2, size=n))).astype(np.float32)
        mo = (g.standard_normal(n, dtype=np.float32) * np.float32(1e-3)).astype(np.float32)
        seed64, stream = int(g.integers(0, 2 ** 62)), int(g.integers(0, 2 ** 31))
        wr, wqr, mr = R.quant_sgd_step(w, gr, mo, lr, mu, *[R.Format(*f) for f in fmts], seed64, stream,
                                       want_wq=mode == "copy", in_place_weights=mode == "in_place", options=R.SgdOptions(*opts))
        what = f"seed {seed} case {case}: n={n} formats={fmts} options={opts} weights={mode} offset={offset}"
        put = lambda a: torch.from_numpy(np.concatenate([np.zeros(offset, np.float32), a])).cuda()[offset:]
        dw, dg, dm = put(w), put(gr), put(mo)
        dq = torch.empty(n, device="cuda") if mode == "copy" else (dw if mode == "in_place" else None)
        Q.quant_sgd_step(dw, dg, dm, lr, mu, *[Q.Format(*f) for f in fmts], seed64, stream, w_q=dq, options=Q.SgdOptions(*opts))
        torch.cuda.synchronize()
        ok = np.isfinite(wr.astype(np.float64)) & np.isfinite(mr.astype(np.float64))      # NaN payloads made by arithmetic are unspecified
        assert_bit_equal(dm.cpu().numpy()[ok], mr[ok], what + ": momentum")
        assert_bit_equal(dw.cpu().numpy()[ok], wr[ok], what + ": weights")
        if mode == "copy":
            assert_bit_equal(dq.cpu().numpy()[ok], wqr[ok], what + ": quantized weights")


def test_random_views_of_a_large_tensor():
    """Seeded random views [outer, nblocks, inner] of 4 to 32 Mi elements (the sizes at which the
    single-pass, block-by-block, flat, column and two-pass forms are chosen), against the oracle."""
    g = np.random.Generator(np.random.PCG64(77))
    total = 1 << 25
    done = 0
    while done < 16:
        a = g.uniform(0, 25)
        b = g.uniform(0, 25 - a)
        if g.integers(0, 3) == 0:
            a = 0.0
        outer = max(1, int(round(2 ** a * g.uniform(0.7, 1.3))))
        nblocks = max(1, int(round(2 ** b * g.uniform(0.7, 1.3))))
        inner = max(1, total // (outer * nblocks))
        if g.integers(0, 2) == 0:
            inner = max(4, inner // 4 * 4)
        n = outer * nblocks * inner
        if n > total or n < total // 8:
            continue
        rounding, offset = int(g.integers(0, 4)), int(g.choice([0, 0, 1]))
        scale = np.exp2(g.integers(-10, 10, size=nblocks)).astype(np.float32)
        x = (g.standard_normal((outer, nblocks, inner), dtype=np.float32) * scale[None, :, None]).astype(np.float32).reshape(-1)
        want = R.block_quantize(x, outer, nblocks, inner, 8, rounding, 0, 5, done)
        d = torch.from_numpy(np.concatenate([np.zeros(offset, np.float32), x])).cuda()[offset:]
        got = Q.block_quantize(d, outer, nblocks, inner, 8, rounding, 0, 5, done)
        torch.cuda.synchronize()
        assert_bit_equal(got.cpu().numpy(), want.reshape(-1), f"[{outer},{nblocks},{inner}] n={n} mode={rounding} offset={offset}")
        done += 1
