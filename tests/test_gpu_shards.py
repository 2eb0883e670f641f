"""Shards: a tensor quantized piece by piece (each piece with its position in the whole tensor)
must equal the oracle's result on the whole tensor, bit for bit; blocks that span pieces go through
the block maxima of all pieces."""
import numpy as np
import pytest

from helpers import assert_bit_equal

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import qsim_ref as R                          # noqa: E402
from paper_1910_04540_amd import binding as Q             # noqa: E402
from paper_1910_04540_amd import workloads as W           # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()


def pieces(n, cuts):
    edges = [0] + [c for c in cuts if 0 < c < n] + [n]
    return list(zip(edges[:-1], edges[1:]))


@pytest.mark.parametrize("rounding", [R.RN_EVEN, R.STOCHASTIC])
def test_elementwise_shards(rounding):
    n = 100003
    x = W.lognormal_gradients(n, seed=11, overflow_fraction=0.01)
    want_fixed = R.fixed_quantize(x, 8, 6, rounding, R.SATURATE, 1234, 3)
    want_float = R.float_quantize(x, 5, 2, rounding, R.SATURATE | R.SUBNORMAL, 1234, 3)
    got_fixed, got_float = np.empty_like(x), np.empty_like(x)
    for k, (lo, hi) in enumerate(pieces(n, [4096, 4100, 50000, 99996])):
        pad = np.zeros(1, np.float32)
        # every other shard sits at a misaligned address (the dword path)
        d = dev(np.concatenate([pad, x[lo:hi]]))[1:] if k % 2 else dev(x[lo:hi])
        got_fixed[lo:hi] = host(Q.fixed_quantize(d, 8, 6, rounding, Q.SATURATE, 1234, 3, index0=lo))
        got_float[lo:hi] = host(Q.float_quantize(d, 5, 2, rounding, Q.SATURATE | Q.SUBNORMAL, 1234, 3, index0=lo))
    assert_bit_equal(got_fixed, want_fixed, "fixed point in shards")
    assert_bit_equal(got_float, want_float, "floating point in shards")


def test_elementwise_shard_far_into_a_tensor():
    """The counter carries into its upper word: a shard that starts at element 2^34 - 8."""
    n, index0 = 64, (1 << 34) - 8
    x = W.uniform_with_outliers(n, seed=5)
    want = np.empty_like(x)
    for i in range(n):
        want[i] = R.fixed_scalar(x[i], 8, 6, R.STOCHASTIC, R.SATURATE, R.random_word(9, 2, 0, index0 + i))
    assert_bit_equal(host(Q.fixed_quantize(dev(x), 8, 6, Q.STOCHASTIC, Q.SATURATE, 9, 2, index0=index0)), want, "offset 2^34 - 8")


@pytest.mark.parametrize("rows,cols,cuts", [(40, 1000, [7, 8, 31]), (24, 1001, [4, 20]), (6, 40000, [1, 5]), (300, 48, [100])])
def test_block_rows_in_shards(rows, cols, cuts):
    x = W.row_scaled_matrix(rows, cols, seed=rows)
    want = R.block_quantize(x, 1, rows, cols, 8, R.STOCHASTIC, 0, 77, 1)
    got = np.empty_like(x)
    for lo, hi in pieces(rows, cuts):
        got[lo:hi] = host(Q.block_quantize(dev(x[lo:hi]), 1, hi - lo, cols, 8, Q.STOCHASTIC, 0, 77, 1, index0=lo * cols))
    assert_bit_equal(got, want, f"{rows} rows of {cols} in shards of whole rows")


@pytest.mark.parametrize("n,cuts", [(300001, [4096, 100000, 250000]), (5000, [2500]), (2 ** 22 + 4, [2 ** 21]), (16, [8])])
@pytest.mark.parametrize("rounding", [R.RN_EVEN, R.STOCHASTIC])
def test_whole_tensor_block_split_over_shards(n, cuts, rounding):
    x = W.row_scaled_matrix(1, n, seed=n % 97).reshape(-1)
    x[n // 3] = np.float32(-7.5e3)                              # the maximum sits in one shard only
    want = R.block_quantize(x, 1, 1, n, 8, rounding, 0, 5, 9)
    shards = [(lo, dev(x[lo:hi])) for lo, hi in pieces(n, cuts)]
    maxima = [Q.block_max(d, 1, 1, d.numel()) for _, d in shards]
    total = maxima[0]
    for m in maxima[1:]:
        total = torch.maximum(total, m)                          # what a max-all-reduce would leave on every GPU
    assert int(total.item()) == int(np.abs(x).max().view(np.uint32))
    got = np.empty_like(x)
    for lo, d in shards:
        got[lo:lo + d.numel()] = host(Q.block_quantize_with_max(d, 1, 1, d.numel(), 8, total, rounding, 0, 5, 9, index0=lo))
    assert_bit_equal(got, want, f"one block of {n} elements split at {cuts}")


def test_blocks_along_a_dimension_sharded_over_the_batch():
    """[outer, nblocks, inner] with the batch (outer) dimension split: every block spans all shards."""
    outer, nblocks, inner = 12, 5, 36
    x = W.lognormal_gradients((outer, nblocks, inner), seed=2)
    want = R.block_quantize(x, outer, nblocks, inner, 8, R.STOCHASTIC, R.SYMMETRIC, 3, 4)
    parts = [(lo, hi, dev(x[lo:hi])) for lo, hi in pieces(outer, [4, 5])]
    total = None
    for lo, hi, d in parts:
        m = Q.block_max(d, hi - lo, nblocks, inner)
        total = m if total is None else torch.maximum(total, m)
    ref_max = np.abs(x).max(axis=(0, 2)).astype(np.float32).view(np.uint32)
    assert np.array_equal(host(total).view(np.uint32), ref_max)
    got = np.empty_like(x)
    for lo, hi, d in parts:
        got[lo:hi] = host(Q.block_quantize_with_max(d, hi - lo, nblocks, inner, 8, total, Q.STOCHASTIC, Q.SYMMETRIC, 3, 4,
                                                    index0=lo * nblocks * inner)).reshape(hi - lo, nblocks, inner)
    assert_bit_equal(got, want, "blocks along dim 1, batch sharded")


@pytest.mark.parametrize("shape", [(1, 1, 70000), (1, 33, 1000), (1, 7, 16385), (1, 5, 999), (9, 4, 50), (3, 2, 5000),
                                   (1, 100, 8)])
def test_block_max_then_quantize_equals_the_fused_call(shape):
    outer, nblocks, inner = shape
    x = W.lognormal_gradients(shape, seed=sum(shape))
    n = x.size
    if outer == 1:
        x = x.reshape(-1)[: n - inner // 3].copy()                # a short last block
    d = dev(x.reshape(-1))
    maxima = Q.block_max(d, outer, nblocks, inner)
    flat = np.zeros(outer * nblocks * inner, np.float32)
    flat[: x.size] = np.abs(x.reshape(-1))
    ref_max = flat.reshape(outer, nblocks, inner).max(axis=(0, 2)).view(np.uint32)
    assert np.array_equal(host(maxima).view(np.uint32), ref_max)
    for rounding in (R.RN_AWAY, R.STOCHASTIC):
        want = R.block_quantize(x, outer, nblocks, inner, 6, rounding, 0, 1, 2).reshape(-1)
        got = host(Q.block_quantize_with_max(d, outer, nblocks, inner, 6, maxima, rounding, 0, 1, 2))
        assert_bit_equal(got, want, f"{shape} rounding {rounding}")


def test_sgd_step_in_shards():
    n = 256 * 37 + 19
    w, g, m = W.sgd_state(n)
    fo = [R.Format(R.KIND_FLOAT, 5, 2, R.STOCHASTIC, 3), R.Format(R.KIND_FIXED, 16, 12, R.STOCHASTIC, 1),
          R.Format(R.KIND_BLOCK, 8, 256, R.STOCHASTIC, 0)]
    fq = [Q.Format(f.kind, f.a, f.b, f.rounding, f.flags) for f in fo]
    wr, wqr, mr = R.quant_sgd_step(w, g, m, 0.1, 0.9, fo[0], fo[1], fo[2], 1234, 6, options=R.SgdOptions(1e-3, 0.0, 1))
    gw, gq, gm = np.empty_like(w), np.empty_like(w), np.empty_like(w)
    for lo, hi in pieces(n, [256, 256 * 20]):
        dw, dg, dm, dq = dev(w[lo:hi]), dev(g[lo:hi]), dev(m[lo:hi]), torch.empty(hi - lo, device="cuda")
        Q.quant_sgd_step(dw, dg, dm, 0.1, 0.9, fq[0], fq[1], fq[2], 1234, 6, w_q=dq, options=Q.SgdOptions(1e-3, 0.0, 1),
                         index0=lo)
        gw[lo:hi], gq[lo:hi], gm[lo:hi] = host(dw), host(dq), host(dm)
    assert_bit_equal(gm, mr, "momentum in shards")
    assert_bit_equal(gw, wr, "weights in shards")
    assert_bit_equal(gq, wqr, "quantized weights in shards")
