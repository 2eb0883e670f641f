"""Parity of the HIP kernels with the CPU oracle, bit for bit, through the C-ABI binding.

Every case feeds the same seeded array to both sides.  Small cases span several tiles and a ragged
tail; the full-size cases are the benchmark's workloads in the launch configuration it times.
"""
import os

import numpy as np
import pytest

from helpers import assert_bit_equal

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from oracle import qsim_ref as R                                    # noqa: E402
from paper_1910_04540_amd import binding as Q                       # noqa: E402
from paper_1910_04540_amd import workloads as W                     # noqa: E402

RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC = 0, 1, 2, 3
SATURATE, SUBNORMAL, SYMMETRIC = 1, 2, 4
MODES = [RN_EVEN, RN_AWAY, RN_ZERO, STOCHASTIC]
THREADS = min(16, os.cpu_count() or 1)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run them with -m gpu on an MI355X box)")
    Q.lib()


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


SPECIALS = np.array([0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x007FFFFF, 0x807FFFFF, 0x00800000, 0x00400000,
                     0x7F7FFFFF, 0xFF7FFFFF, 0x7F800000, 0xFF800000, 0x7FC00000, 0xFFC12345, 0x7F800001, 0x3F800000,
                     0x3F7FFFFF, 0x3F800001, 0x33800000, 0x33FFFFFF, 0x4B800000, 0xCB7FFFFF],
                    dtype=np.uint32).view(np.float32)


def probe_array(n, seed):
    """Mixed-scale values, a normal body and the special encodings; n is ragged on purpose."""
    parts = [W.mixed_scales(n // 2, seed=seed), W.normal_tensor(n - n // 2 - SPECIALS.size, seed=seed + 1), SPECIALS]
    x = np.concatenate(parts).astype(np.float32)
    return x[np.random.Generator(np.random.PCG64(seed)).permutation(x.size)]


# ------------------------------------------------------------------------------------------------
# fixed point
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("rounding", MODES)
@pytest.mark.parametrize("wl,fl,flags", [(8, 6, SATURATE), (8, 6, 0), (16, 12, SATURATE), (24, 20, SATURATE),
                                         (24, 10, SATURATE | SYMMETRIC), (1, 0, SATURATE), (2, 1, SATURATE),
                                         (12, -3, SATURATE), (8, 149, SATURATE), (8, 140, 0), (10, -118, SATURATE),
                                         (4, -100, 0), (24, 149, SATURATE), (5, 30, SATURATE | SYMMETRIC)])
def test_fixed_small(wl, fl, flags, rounding):
    n = 4 * 1024 * 3 + 4 * 77 + 3
    x = probe_array(n, seed=100 + wl)
    # some values at the scale of the format's own grid
    x[: n // 4] = (W.uniform_with_outliers(n // 4, seed=7) * np.float32(2.0 ** (wl - 3 - fl))).astype(np.float32)
    want = R.fixed_quantize(x, wl, fl, rounding, flags, seed=1234, stream_id=9, threads=THREADS)
    got = host(Q.fixed_quantize(dev(x), wl, fl, rounding, flags, seed=1234, stream_id=9))
    assert_bit_equal(got, want, f"fixed({wl},{fl}) flags {flags} mode {rounding}")


@pytest.mark.parametrize("n", [0, 1, 2, 3, 4, 5, 255, 1023, 1024, 1025, 4096, 4097, 4 * 1024 * 2 + 1])
def test_fixed_sizes_alignment_and_inplace(n):
    x = W.uniform_with_outliers(n + 8, seed=n + 1)
    for off in (0, 1, 3):
        xs = x[off:off + n]
        want = R.fixed_quantize(xs, 8, 6, STOCHASTIC, SATURATE, seed=5, stream_id=1)
        d = dev(x)
        view = d[off:off + n]
        got = host(Q.fixed_quantize(view, 8, 6, STOCHASTIC, SATURATE, seed=5, stream_id=1))
        assert_bit_equal(got, want, f"n={n} offset={off}")
        # in place, and nothing outside the view is touched
        Q.fixed_quantize(view, 8, 6, STOCHASTIC, SATURATE, seed=5, stream_id=1, out=view)
        full = host(d)
        assert_bit_equal(full[off:off + n], want, f"in place n={n} offset={off}")
        assert_bit_equal(full[:off], x[:off], "before the view")
        assert_bit_equal(full[off + n:], x[off + n:], "after the view")


def test_indices_beyond_32_bits():
    """2^34 + 4100 elements (64 GiB, quantized in place): element indices need 35 bits and the Philox
    counter's high word becomes non-zero.  Checked on windows around the 2^32 and 2^34 boundaries and
    at both ends against the oracle, which is given the window's offset."""
    n = (1 << 34) + 4100
    free, _ = torch.cuda.mem_get_info()
    if free < n * 4 + (4 << 30):
        pytest.skip("not enough free device memory for a 64 GiB tensor")
    base = dev(W.uniform_with_outliers(1 << 26, seed=5))
    x = torch.empty(n, device="cuda")
    for k in range(n // base.numel()):
        x[k * base.numel():(k + 1) * base.numel()] = base
    x[(n // base.numel()) * base.numel():] = base[: n % base.numel()]
    x[(1 << 32) - 5: (1 << 32) + 5] = torch.linspace(-2.5, 2.5, 10, device="cuda")
    windows = [(0, 2048), ((1 << 32) - 1000, 2000), ((1 << 33) + 12345, 1111), ((1 << 34) - 3000, 3000 + 4100)]
    before = [(o, host(x[o:o + c])) for o, c in windows]
    Q.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=1234, stream_id=3, out=x)
    lib = R.lib()
    import ctypes
    for o, inp in before:
        want = np.empty_like(inp)
        fp = ctypes.POINTER(ctypes.c_float)
        assert lib.qsim_ref_fixed_quantize_at(inp.ctypes.data_as(fp), want.ctypes.data_as(fp), inp.size, o, 8, 6,
                                              STOCHASTIC, SATURATE, 1234, 3) == 0
        assert_bit_equal(host(x[o:o + inp.size]), want, f"window at {o}")
    del x
    torch.cuda.empty_cache()


def test_many_small_blocks_beyond_32_bits():
    """2^32 + 64 elements in chunks of 16 (268 million blocks, a grid folded over two dimensions),
    nearest rounding in place; windows of whole chunks against the oracle."""
    n = (1 << 32) + 64
    free, _ = torch.cuda.mem_get_info()
    if free < n * 4 + (4 << 30):
        pytest.skip("not enough free device memory for a 16 GiB tensor")
    g0 = np.random.Generator(np.random.PCG64(2))
    base = dev((W.normal_tensor(1 << 24, seed=9) * np.exp2(g0.integers(-20, 20, 1 << 24))).astype(np.float32))
    x = torch.empty(n, device="cuda")
    for k in range(n // base.numel()):
        x[k * base.numel():(k + 1) * base.numel()] = base
    x[(n // base.numel()) * base.numel():] = base[: n % base.numel()]
    windows = [(0, 1600), ((1 << 31) - 160, 320), ((1 << 32) - 1600, 1664)]
    before = [(o, host(x[o:o + c])) for o, c in windows]
    Q.block_quantize(x, 1, n // 16, 16, 8, RN_EVEN, out=x)
    for o, inp in before:
        assert_bit_equal(host(x[o:o + inp.size]), R.block_quantize(inp, 1, inp.size // 16, 16, 8, RN_EVEN), f"window at {o}")
    del x
    torch.cuda.empty_cache()


def test_blocks_along_a_dimension_beyond_32_bits():
    """[16, 4200, 65536] = 2^32 + 1.1e8 elements with one block per middle index (64 slices of 16 Ki
    each, workgroups of a block meeting among themselves), nearest rounding in place; three blocks
    gathered from the GPU and checked against the oracle."""
    outer, nblocks, inner = 16, 4200, 65536
    n = outer * nblocks * inner
    free, _ = torch.cuda.mem_get_info()
    if free < n * 4 + (4 << 30):
        pytest.skip("not enough free device memory for an 18 GiB tensor")
    x = torch.randn(n, device="cuda")
    view = x.view(outer, nblocks, inner)
    view *= torch.exp2(torch.randint(-12, 12, (nblocks,), device="cuda").float())[None, :, None]
    picks = [0, 2099, nblocks - 1]
    before = {b: host(view[:, b, :]).copy() for b in picks}
    Q.block_quantize(x, outer, nblocks, inner, 8, RN_EVEN, out=x)
    for b in picks:
        want = R.block_quantize(before[b], outer, 1, inner, 8, RN_EVEN)
        assert_bit_equal(host(view[:, b, :]).reshape(-1), want.reshape(-1), f"block {b}")
    del x, view
    torch.cuda.empty_cache()


def test_seed_and_stream_select_the_words():
    x = dev(W.uniform_with_outliers(1 << 14, seed=3))
    a = host(Q.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=1, stream_id=0))
    assert np.array_equal(a, host(Q.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=1, stream_id=0)))
    assert not np.array_equal(a, host(Q.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=2, stream_id=0)))
    assert not np.array_equal(a, host(Q.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=1, stream_id=1)))
    big = (1 << 63) + 12345
    want = R.fixed_quantize(host(x), 8, 6, STOCHASTIC, SATURATE, seed=big, stream_id=0xFFFFFFFF)
    assert_bit_equal(host(Q.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=big, stream_id=0xFFFFFFFF)), want, "64-bit seed")


# ------------------------------------------------------------------------------------------------
# floating point
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("rounding", MODES)
@pytest.mark.parametrize("flags", [0, SATURATE, SUBNORMAL, SATURATE | SUBNORMAL])
@pytest.mark.parametrize("e,m", [(5, 2), (5, 10), (8, 7), (4, 3), (2, 1), (8, 23), (8, 1), (3, 22), (6, 9), (7, 23), (2, 23)])
def test_float_small(e, m, flags, rounding):
    n = 4 * 1024 * 2 + 4 * 13 + 1
    bias = (1 << (e - 1)) - 1
    x = probe_array(n, seed=200 + e * 31 + m)
    x[: n // 3] = W.mixed_scales(n // 3, seed=5, lo_exp=-bias - m - 6, hi_exp=min(bias + 5, 128))
    want = R.float_quantize(x, e, m, rounding, flags, seed=99, stream_id=4, threads=THREADS)
    got = host(Q.float_quantize(dev(x), e, m, rounding, flags, seed=99, stream_id=4))
    assert_bit_equal(got, want, f"float({e},{m}) flags {flags} mode {rounding}")


@pytest.mark.parametrize("e,m,flags", [(5, 10, SATURATE | SUBNORMAL), (5, 10, 0), (8, 7, SATURATE | SUBNORMAL), (8, 7, SATURATE),
                                       (5, 2, SATURATE | SUBNORMAL), (5, 2, SATURATE)])
@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
def test_float_every_exponent_and_dropped_bit_class(e, m, flags, rounding):
    """Every (sign, exponent, kept mantissa) of fp32 with the low-bit patterns that decide a
    rounding: 8 Mi encodings per format, NaN and Inf included."""
    x = W.all_exponents_probe(23 - m)
    want = R.float_quantize(x, e, m, rounding, flags, seed=3, threads=THREADS)
    got = host(Q.float_quantize(dev(x), e, m, rounding, flags, seed=3))
    assert_bit_equal(got, want, f"float({e},{m}) flags {flags} mode {rounding}")


@pytest.mark.parametrize("kind,a,b,rounding,flags", [
    ("float", 5, 10, RN_EVEN, 3),        # per-element grid, nearest
    ("float", 5, 2, STOCHASTIC, 3),      # per-element grid, stochastic
    ("float", 8, 7, STOCHASTIC, 3),      # constant mask, stochastic
    ("float", 5, 2, RN_EVEN, 1),         # constant mask, flush to zero
    ("float", 8, 7, RN_AWAY, 0),         # constant mask, flush with the fp32-denormal side path, no saturation
    ("fixed", 8, 6, STOCHASTIC, 1),      # fixed grid, saturating
    ("fixed", 12, 20, RN_ZERO, 0),       # fixed grid, open range
    ("fixed", 16, 12, STOCHASTIC, 1),    # the momentum format of the optimizer workload
    ("float", 5, 10, RN_EVEN, 0),        # the gradient workload's format with flags clear: flush to zero, open range
    ("float", 5, 2, RN_EVEN, 3),         # the first workload's format with gradual underflow
])
def test_exhaustive_all_fp32_encodings(kind, a, b, rounding, flags):
    """All 2^32 fp32 encodings (NaN and Inf included) through one format, against the oracle."""
    chunk = 1 << 26
    for start in range(0, 1 << 32, chunk):
        x = np.arange(start, start + chunk, dtype=np.uint64).astype(np.uint32).view(np.float32)
        if kind == "float":
            want = R.float_quantize(x, a, b, rounding, flags, seed=1234, threads=THREADS)
            got = host(Q.float_quantize(dev(x), a, b, rounding, flags, seed=1234))
        else:
            want = R.fixed_quantize(x, a, b, rounding, flags, seed=1234, threads=THREADS)
            got = host(Q.fixed_quantize(dev(x), a, b, rounding, flags, seed=1234))
        assert_bit_equal(got, want, f"{kind}({a},{b}) chunk {start:#x}")


# ------------------------------------------------------------------------------------------------
# block floating point
# ------------------------------------------------------------------------------------------------
def _block_case(x, outer, nblocks, inner, wl, rounding, flags=0, seed=1234, stream_id=2):
    want = R.block_quantize(x, outer, nblocks, inner, wl, rounding, flags, seed, stream_id)
    got = host(Q.block_quantize(dev(x), outer, nblocks, inner, wl, rounding, flags, seed, stream_id))
    assert_bit_equal(got, want, f"block [{outer},{nblocks},{inner}] wl {wl} mode {rounding} flags {flags}")


@pytest.mark.parametrize("rounding", MODES)
@pytest.mark.parametrize("wl", [8, 2, 24, 5])
def test_block_rows(wl, rounding):
    x = W.row_scaled_matrix(96, 1024 + 256, seed=3)
    x[7] = 0.0
    x[8] = np.float32(1e-41)
    x[9, 5] = np.float32(3.3e38)
    x[10, 17] = np.float32(-3.4e38)
    _block_case(x, 1, 96, 1280, wl, rounding)
    _block_case(x, 1, 96, 1280, wl, rounding, flags=SYMMETRIC)


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("rows,cols", [(3, 5000), (1, 70001), (600, 7), (40, 333), (1000, 64), (17, 4096), (2, 65536 + 4)])
def test_block_row_shapes(rows, cols, rounding):
    x = W.row_scaled_matrix(rows, cols, seed=rows + cols)
    _block_case(x, 1, rows, cols, 8, rounding)


@pytest.mark.parametrize("rounding", [RN_AWAY, STOCHASTIC])
@pytest.mark.parametrize("rows,cols,short", [(70000, 1, 0), (50001, 2, 1), (40000, 3, 2), (30000, 5, 0), (20000, 10, 3),
                                             (9000, 27, 0), (700, 1001, 500), (50, 4098, 0), (9, 8190, 1), (5, 16377, 0),
                                             (5, 16378, 7), (3, 16379, 0), (2, 16383, 16000), (3000, 4095, 0)])
def test_block_lengths_that_are_not_whole_groups(rows, cols, short, rounding):
    """Contiguous blocks whose length is not a multiple of four, so that the tensor's groups of four
    straddle blocks and workgroups share their first and last group; a short last block; the same
    from a misaligned address and in place."""
    n = rows * cols - short
    x = W.row_scaled_matrix(rows, cols, seed=rows + cols).reshape(-1)[:n].copy()
    x[n // 2] = np.float32(-1.0e30)
    want = R.block_quantize(x, 1, rows, cols, 8, rounding, 0, 21, 5)
    assert_bit_equal(host(Q.block_quantize(dev(x), 1, rows, cols, 8, rounding, 0, 21, 5)), want, f"{rows} blocks of {cols}")
    pad = dev(np.concatenate([np.zeros(3, np.float32), x, np.zeros(2, np.float32)]))
    view = pad[3:3 + n]
    assert_bit_equal(host(Q.block_quantize(view, 1, rows, cols, 8, rounding, 0, 21, 5)), want, "from a misaligned address")
    Q.block_quantize(view, 1, rows, cols, 8, rounding, 0, 21, 5, out=view)
    full = host(pad)
    assert_bit_equal(full[3:3 + n], want, "in place")
    assert not full[:3].any() and not full[3 + n:].any()


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("rows,cols,short", [(5, 70001, 0), (40, 29799, 0), (7, 29799, 29000), (3, 1342177, 5), (2, 4000003, 1),
                                             (9, 16386, 16385), (3, 65536, 0), (1, 2000001, 0)])
def test_block_long_rows_of_odd_length(rows, cols, short, rounding):
    """Contiguous blocks longer than one workgroup holds whose length is not a multiple of four, or
    that start at a misaligned address: single pass block by block over the tensor's own groups of
    four (up to 4 Mi elements per block, two passes beyond); a short last block; in place."""
    n = rows * cols - short
    x = W.row_scaled_matrix(rows, cols, seed=rows + cols).reshape(-1)[:n].copy()
    x[cols - 1] = np.float32(3.0e30)                   # the first block's maximum in its very last element
    want = R.block_quantize(x, 1, rows, cols, 8, rounding, 0, 21, 5)
    pad = dev(np.zeros(n + 8, np.float32))
    for off in (0, 1, 2, 3):
        view = pad[off:off + n]
        view.copy_(torch.from_numpy(x))
        out = torch.full((n + 8,), 7.0, device="cuda")
        Q.block_quantize(view, 1, rows, cols, 8, rounding, 0, 21, 5, out=out[off:off + n])
        assert_bit_equal(host(out[off:off + n]), want, f"{rows} blocks of {cols} less {short}, offset {off}")
        assert bool((out[:off] == 7.0).all()) and bool((out[off + n:] == 7.0).all()), f"offset {off}: wrote outside"
    Q.block_quantize(view, 1, rows, cols, 8, rounding, 0, 21, 5, out=view)
    assert_bit_equal(host(view), want, "in place")


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("rows,cols,short", [(600, 20000, 0), (1100, 16388, 100), (270, 65536, 0), (530, 32772, 5000)])
def test_block_many_long_rows(rows, cols, short, rounding):
    """More rows of 16 Ki to 64 Ki elements than the chip holds at once: one 1024-thread workgroup per row."""
    n = rows * cols - short
    x = W.row_scaled_matrix(rows, cols, seed=rows).reshape(-1)[:n].copy()
    want = R.block_quantize(x, 1, rows, cols, 8, rounding, 0, 8, 1)
    d = dev(x)
    assert_bit_equal(host(Q.block_quantize(d, 1, rows, cols, 8, rounding, 0, 8, 1)), want, f"{rows} rows of {cols}")
    Q.block_quantize(d, 1, rows, cols, 8, rounding, 0, 8, 1, out=d)
    assert_bit_equal(host(d), want, "in place")


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("n", [1, 3, 1000, 8192, 8193, 100003, (1 << 20) + 4, 3 * (1 << 20) + 1])
def test_block_whole_tensor(n, rounding):
    x = W.row_scaled_matrix(1, n, seed=n % 97)
    _block_case(x, 1, 1, n, 8, rounding)


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("n,L", [(4096, 256), (4096 + 100, 256), (10000, 16), (999, 64), (70000, 1024), (300000, 32768)])
def test_block_contiguous_chunks(n, L, rounding):
    x = (W.normal_tensor(n, seed=n) * np.exp2(np.random.Generator(np.random.PCG64(n)).integers(-12, 12, n))).astype(np.float32)
    _block_case(x, 1, (n + L - 1) // L, L, 8, rounding)


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("shape,dim", [((6, 5, 7), 1), ((6, 5, 7), 2), ((16, 32, 64), 1), ((64, 20, 36), 1),
                                       ((300, 40), 1), ((8, 3, 1024), 1), ((2, 2, 40000), 1), ((50, 8, 3), 1),
                                       ((40, 6, 6), 1), ((33, 1000, 12), 1), ((1030, 2052), 1), ((5, 64, 14, 14), 1),
                                       ((3, 2, 4, 2), 2), ((70000, 4), 1), ((17, 2, 2), 1)])
def test_block_over_an_inner_dimension(shape, dim, rounding):
    g = np.random.Generator(np.random.PCG64(int(np.prod(shape))))
    x = (g.standard_normal(shape) * np.exp2(g.integers(-10, 10, size=shape))).astype(np.float32)
    outer = int(np.prod(shape[:dim]))
    inner = int(np.prod(shape[dim + 1:]))
    _block_case(x, outer, shape[dim], inner, 8, rounding)


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("outer,nblocks,inner", [(5000, 3, 300), (1048577, 5, 1), (9000, 4096, 1), (300000, 3, 7),
                                                 (3, 32768, 1), (600, 128, 256), (70001, 1, 3), (2, 1, 1), (100001, 255, 1), (200, 2, 16385),
                                                 (90, 61440, 1), (70, 4, 15360), (50, 3, 20479)])
def test_block_short_rows_many_of_them(outer, nblocks, inner, rounding):
    """Blocks along an inner dimension with rows of at most 60 Ki elements: the flat walk with the
    block table in LDS, several steps per workgroup, ragged tails, also from a misaligned address
    and in place."""
    g = np.random.Generator(np.random.PCG64(outer + nblocks + inner))
    n = outer * nblocks * inner
    scale = np.exp2(g.integers(-10, 10, size=nblocks)).astype(np.float32)
    x = (g.standard_normal((outer, nblocks, inner), dtype=np.float32) * scale[None, :, None]).astype(np.float32)
    x.reshape(-1)[g.integers(0, n)] = np.float32(3.0e33)
    want = R.block_quantize(x, outer, nblocks, inner, 8, rounding, 0, 17, 3).reshape(-1)
    assert_bit_equal(host(Q.block_quantize(dev(x.reshape(-1)), outer, nblocks, inner, 8, rounding, 0, 17, 3)), want,
                     f"[{outer},{nblocks},{inner}]")
    pad = dev(np.concatenate([np.zeros(1, np.float32), x.reshape(-1), np.zeros(3, np.float32)]))
    view = pad[1:1 + n]
    Q.block_quantize(view, outer, nblocks, inner, 8, rounding, 0, 17, 3, out=view)
    full = host(pad)
    assert_bit_equal(full[1:1 + n], want, "in place from a misaligned address")
    assert not full[:1].any() and not full[1 + n:].any()


def test_block_misaligned_and_inplace():
    x = W.row_scaled_matrix(1, 50000 + 8, seed=11).reshape(-1)
    for off, n, nb, inner in [(1, 50000, 50, 1000), (3, 49999, 1, 49999), (0, 50000, 50, 1000), (2, 50002, 1, 50002)]:
        xs = x[off:off + n]
        want = R.block_quantize(xs, 1, nb, inner, 8, STOCHASTIC, 0, 5, 6)
        d = dev(x)
        view = d[off:off + n]
        assert_bit_equal(host(Q.block_quantize(view, 1, nb, inner, 8, STOCHASTIC, 0, 5, 6)), want, f"offset {off}")
        Q.block_quantize(view, 1, nb, inner, 8, STOCHASTIC, 0, 5, 6, out=view)
        full = host(d)
        assert_bit_equal(full[off:off + n], want, f"in place offset {off}")
        assert_bit_equal(np.concatenate([full[:off], full[off + n:]]), np.concatenate([x[:off], x[off + n:]]), "outside")


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
def test_block_single_pass_when_the_wait_runs_out(rounding):
    """The single-pass kernel's wait for the other workgroups is bounded; with the bound forced to
    zero from the host every workgroup derives the missing maxima from memory itself and the
    result must still be exact, also in place and with several blocks."""
    Q.set_barrier_wait_us(0)
    try:
        for rows, cols in [(1, 200000), (3, 40000), (1, 16388)]:
            x = W.row_scaled_matrix(rows, cols, seed=rows * 7 + 1)
            x[0, cols // 2] = np.float32(-3.0e4)            # the maximum sits in one slice only
            want = R.block_quantize(x, 1, rows, cols, 8, rounding, 0, 11, 3)
            d = dev(x)
            assert_bit_equal(host(Q.block_quantize(d, 1, rows, cols, 8, rounding, 0, 11, 3)), want, f"{rows}x{cols}")
            Q.block_quantize(d, 1, rows, cols, 8, rounding, 0, 11, 3, out=d)
            assert_bit_equal(host(d), want, f"{rows}x{cols} in place")
    finally:
        Q.set_barrier_wait_us(2000)


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("rows,cols,short", [(300, 70000, 0), (600, 65540, 30000), (40, 1048576, 0), (130, 262148, 100000)])
def test_block_many_rows_that_each_fit_the_registers(rows, cols, short, rounding):
    """More long rows than the chip holds at once, each of at most 64 register-resident slices: the
    workgroups of a row meet among themselves, row after row."""
    n = rows * cols - short
    x = W.row_scaled_matrix(rows, cols, seed=rows + 1).reshape(-1)[:n].copy()
    x[(rows // 2) * cols + cols - 5] = np.float32(9.0e20)        # a maximum that sits in one row's last slice only
    want = R.block_quantize(x, 1, rows, cols, 8, rounding, 0, 4, 2)
    d = dev(x)
    assert_bit_equal(host(Q.block_quantize(d, 1, rows, cols, 8, rounding, 0, 4, 2)), want, f"{rows} rows of {cols}")
    Q.block_quantize(d, 1, rows, cols, 8, rounding, 0, 4, 2, out=d)
    assert_bit_equal(host(d), want, "in place")


def test_block_row_by_row_single_pass_when_the_wait_runs_out():
    """The same with the wait forced to zero: every workgroup derives the maxima of the slices that
    have not been published from memory itself; exact, also in place."""
    Q.set_barrier_wait_us(0)
    try:
        rows, cols = 300, 70000
        x = W.row_scaled_matrix(rows, cols, seed=5).reshape(-1)
        want = R.block_quantize(x, 1, rows, cols, 8, STOCHASTIC, 0, 4, 2)
        d = dev(x)
        assert_bit_equal(host(Q.block_quantize(d, 1, rows, cols, 8, STOCHASTIC, 0, 4, 2)), want, "out of place")
        Q.block_quantize(d, 1, rows, cols, 8, STOCHASTIC, 0, 4, 2, out=d)
        assert_bit_equal(host(d), want, "in place")
    finally:
        Q.set_barrier_wait_us(2000)


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("shape", [(32, 64, 3136), (64, 256, 3136), (64, 3, 65536), (1000, 40, 64), (7, 5, 16388), (3, 1100, 16384)])
def test_block_per_channel_single_pass(shape, rounding):
    """Blocks along an inner dimension made of aligned segments (per-channel blocks of an activation
    tensor): the workgroups of a block meet among themselves, block after block; in place too."""
    outer, nblocks, inner = shape
    g = np.random.Generator(np.random.PCG64(sum(shape)))
    scale = np.exp2(g.integers(-12, 12, size=nblocks)).astype(np.float32)
    x = (g.standard_normal(shape, dtype=np.float32) * scale[None, :, None]).astype(np.float32)
    x[outer - 1, nblocks // 2, inner - 1] = np.float32(-2.0e25)      # a maximum in a block's very last element
    want = R.block_quantize(x, outer, nblocks, inner, 8, rounding, 0, 6, 1).reshape(-1)
    d = dev(x.reshape(-1))
    assert_bit_equal(host(Q.block_quantize(d, outer, nblocks, inner, 8, rounding, 0, 6, 1)), want, f"{shape}")
    Q.block_quantize(d, outer, nblocks, inner, 8, rounding, 0, 6, 1, out=d)
    assert_bit_equal(host(d), want, f"{shape} in place")


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("shape", [(2, 300000, 64), (4, 1000, 4), (2, 5, 1024), (8, 50000, 128), (3, 100001, 100), (2, 1, 4),
                                   (512, 20000, 4), (2, 1000003, 16), (32, 33, 64), (128, 512, 16), (128, 512, 4), (500, 101, 4),
                                   (1000, 7, 8)])
def test_block_short_blocks_along_an_inner_dimension(shape, rounding):
    """Blocks of at most 2048 elements made of whole-group segments: several blocks per workgroup,
    single pass (few outer indices, or a tensor of at most 8 Mi elements)."""
    outer, nblocks, inner = shape
    g = np.random.Generator(np.random.PCG64(sum(shape)))
    scale = np.exp2(g.integers(-12, 12, size=nblocks)).astype(np.float32)
    x = (g.standard_normal(shape, dtype=np.float32) * scale[None, :, None]).astype(np.float32)
    want = R.block_quantize(x, outer, nblocks, inner, 8, rounding, 0, 6, 1).reshape(-1)
    d = dev(x.reshape(-1))
    assert_bit_equal(host(Q.block_quantize(d, outer, nblocks, inner, 8, rounding, 0, 6, 1)), want, f"{shape}")
    Q.block_quantize(d, outer, nblocks, inner, 8, rounding, 0, 6, 1, out=d)
    assert_bit_equal(host(d), want, f"{shape} in place")


@pytest.mark.parametrize("rounding", [RN_EVEN, RN_ZERO, STOCHASTIC])
@pytest.mark.parametrize("shape", [(2, 30000, 154), (2, 1000, 77), (16, 300, 49), (5, 700, 33), (3, 10, 682), (2, 4, 1001), (16, 2048, 49),
                                   (4, 5, 50), (2, 3000, 64), (7, 1, 99), (2, 70000, 9), (12, 4097, 13), (3, 2, 683), (2, 1, 1023),
                                   (16, 9, 127), (2, 100, 1024)])
def test_block_short_blocks_of_odd_segments_along_an_inner_dimension(shape, rounding):
    """Blocks of at most 2048 elements along an inner dimension whose segments are not whole groups,
    or that lie in arrays that start at any element: several blocks per workgroup, each outer index
    one contiguous run walked in the arrays' own groups; one pass.  Every alignment of the arrays;
    neighbouring blocks differ in scale by up to 2^24 and every block's largest value sits at an edge
    of one of its segments, next to a neighbour's elements."""
    outer, nblocks, inner = shape
    g = np.random.Generator(np.random.PCG64(sum(shape)))
    scale = np.exp2(g.integers(-12, 12, size=nblocks)).astype(np.float32)
    x = (g.standard_normal(shape, dtype=np.float32) * scale[None, :, None]).astype(np.float32)
    x[g.integers(0, outer, size=nblocks), np.arange(nblocks), (g.integers(0, 2, size=nblocks) * (inner - 1))] *= np.float32(9.0)
    want = R.block_quantize(x, outer, nblocks, inner, 8, rounding, 0, 6, 1).reshape(-1)
    n = x.size
    pad = dev(np.concatenate([np.zeros(3, np.float32), x.reshape(-1), np.full(5, 1e30, np.float32)]))
    for off in (3, 2, 1, 0):
        view = pad[off:off + n]
        view.copy_(torch.from_numpy(x.reshape(-1)))
        assert_bit_equal(host(Q.block_quantize(view, outer, nblocks, inner, 8, rounding, 0, 6, 1)), want, f"{shape} offset {off}")
    Q.block_quantize(view, outer, nblocks, inner, 8, rounding, 0, 6, 1, out=view)
    assert_bit_equal(host(view), want, f"{shape} in place")
    assert np.all(host(pad[3 + n:]) == np.float32(1e30))             # nothing written behind the arrays


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("shape", [(4, 100003, 1), (46, 5743, 1), (71, 6029, 7), (22, 10601, 14), (631, 3035, 1), (9, 6, 20714),
                                   (5, 3, 4098), (77, 1, 43577), (3, 4, 279622), (40, 72, 1165), (300, 5000, 3),
                                   (2, 3, (1 << 21) + 1), (2, 2, (1 << 21) + 4), (2, 2, (1 << 22) + 1), (3, 2, 2796204)])
def test_block_rows_that_are_not_whole_groups_along_an_inner_dimension(shape, rounding):
    """Blocks along an inner dimension when a row is not a multiple of four elements, or the blocks
    are long and odd: the one-column-per-thread form, the single pass over odd segments (blocks of
    up to 512 workgroups, aligned or not) and, for blocks of more than eight million elements, the
    general two-pass form; one block in several outer pieces is the whole tensor."""
    outer, nblocks, inner = shape
    g = np.random.Generator(np.random.PCG64(sum(shape)))
    scale = np.exp2(g.integers(-12, 12, size=nblocks)).astype(np.float32)
    x = (g.standard_normal(shape, dtype=np.float32) * scale[None, :, None]).astype(np.float32)
    want = R.block_quantize(x, outer, nblocks, inner, 8, rounding, 0, 6, 1).reshape(-1)
    n = x.size
    pad = dev(np.concatenate([np.zeros(2, np.float32), x.reshape(-1), np.zeros(2, np.float32)]))
    for off in (2, 0):
        view = pad[off:off + n]
        if off == 0:
            view.copy_(torch.from_numpy(x.reshape(-1)))
        assert_bit_equal(host(Q.block_quantize(view, outer, nblocks, inner, 8, rounding, 0, 6, 1)), want, f"{shape} offset {off}")
    Q.block_quantize(view, outer, nblocks, inner, 8, rounding, 0, 6, 1, out=view)
    assert_bit_equal(host(view), want, f"{shape} in place")


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("shape", [(70, 5, 129), (70, 7, 132), (70, 3, 130), (70, 2, 131), (130, 5, 65), (128, 6, 729), (7, 11, 4153), (2, 3, 70001),
                                   (33, 64, 3025), (1000, 2, 4001), (130, 300, 65), (3, 2, 1048577), (9, 5, 3136), (3, 5, 65)])
def test_block_per_channel_single_pass_with_odd_segments(shape, rounding):
    """Blocks along an inner dimension made of segments of any length, at every alignment of the
    arrays (single pass above 128 elements per segment, the flat or column form below): the first and last group of a segment hold a neighbouring block's
    elements, which must neither count for the maximum nor be written.  Neighbouring blocks differ
    in scale by up to 2^24 and each block's maximum sits at the edge of one of its segments."""
    outer, nblocks, inner = shape
    g = np.random.Generator(np.random.PCG64(sum(shape)))
    scale = np.exp2(g.integers(-12, 12, size=nblocks)).astype(np.float32)
    x = (g.standard_normal(shape, dtype=np.float32) * scale[None, :, None]).astype(np.float32)
    for b in range(min(nblocks, 64)):
        x[g.integers(outer), b, (0, inner - 1)[b % 2]] = np.float32(37.0) * scale[b] * np.float32((-1) ** b)
    want = R.block_quantize(x, outer, nblocks, inner, 8, rounding, 0, 6, 1).reshape(-1)
    n = x.size
    pad = dev(np.zeros(n + 8, np.float32))
    for off in (0, 1, 2, 3):
        view = pad[off:off + n]
        view.copy_(torch.from_numpy(x.reshape(-1)))
        out = torch.full((n + 8,), 7.0, device="cuda")
        Q.block_quantize(view, outer, nblocks, inner, 8, rounding, 0, 6, 1, out=out[off:off + n])
        assert_bit_equal(host(out[off:off + n]), want, f"{shape} offset {off}")
        assert bool((out[:off] == 7.0).all()) and bool((out[off + n:] == 7.0).all()), f"{shape} offset {off}: wrote outside"
    Q.block_quantize(view, outer, nblocks, inner, 8, rounding, 0, 6, 1, out=view)
    assert_bit_equal(host(view), want, f"{shape} in place")


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
@pytest.mark.parametrize("shape", [(128, 16, 256), (100, 9, 256), (4, 6, 16000), (65, 700, 252), (2, 3, 32768), (17, 2, 3852)])
def test_block_per_channel_one_large_workgroup_per_block(shape, rounding):
    """Blocks along an inner dimension of 16 Ki to 64 Ki elements: one workgroup of 512 or 1024
    threads holds a block alone (full, partly filled, and exactly full workgroups)."""
    outer, nblocks, inner = shape
    g = np.random.Generator(np.random.PCG64(sum(shape)))
    scale = np.exp2(g.integers(-12, 12, size=nblocks)).astype(np.float32)
    x = (g.standard_normal(shape, dtype=np.float32) * scale[None, :, None]).astype(np.float32)
    x[outer - 1, nblocks - 1, inner - 1] = np.float32(7.0e22)          # a maximum in the tensor's very last element
    want = R.block_quantize(x, outer, nblocks, inner, 8, rounding, 0, 6, 1).reshape(-1)
    d = dev(x.reshape(-1))
    assert_bit_equal(host(Q.block_quantize(d, outer, nblocks, inner, 8, rounding, 0, 6, 1)), want, f"{shape}")
    Q.block_quantize(d, outer, nblocks, inner, 8, rounding, 0, 6, 1, out=d)
    assert_bit_equal(host(d), want, f"{shape} in place")


def test_block_per_channel_single_pass_with_odd_segments_when_the_wait_runs_out():
    Q.set_barrier_wait_us(0)
    try:
        for shape in [(128, 6, 729), (2, 3, 70001)]:
            x = W.lognormal_gradients(shape, seed=11)
            want = R.block_quantize(x, *shape, 8, STOCHASTIC, 0, 6, 1).reshape(-1)
            pad = dev(np.concatenate([np.zeros(1, np.float32), x.reshape(-1)]))
            d = pad[1:]
            assert_bit_equal(host(Q.block_quantize(d, *shape, 8, STOCHASTIC, 0, 6, 1)), want, f"{shape} out of place")
            Q.block_quantize(d, *shape, 8, STOCHASTIC, 0, 6, 1, out=d)
            assert_bit_equal(host(d), want, f"{shape} in place")
    finally:
        Q.set_barrier_wait_us(2000)


def test_block_per_channel_single_pass_when_the_wait_runs_out():
    Q.set_barrier_wait_us(0)
    try:
        shape = (32, 64, 3136)
        x = W.lognormal_gradients(shape, seed=9)
        want = R.block_quantize(x, *shape, 8, STOCHASTIC, 0, 6, 1).reshape(-1)
        d = dev(x.reshape(-1))
        assert_bit_equal(host(Q.block_quantize(d, *shape, 8, STOCHASTIC, 0, 6, 1)), want, "out of place")
        Q.block_quantize(d, *shape, 8, STOCHASTIC, 0, 6, 1, out=d)
        assert_bit_equal(host(d), want, "in place")
    finally:
        Q.set_barrier_wait_us(2000)


KEPT_SHAPES = [(1, 1, 4096 * 4096), (1, 3, 2000000), (1, 300, 70000), (64, 96, 3136), (128, 6, 729), (40, 64, 3025)]


@pytest.mark.parametrize("shape", KEPT_SHAPES)
def test_block_single_pass_with_a_kept_workspace(shape):
    """A caller keeps one zero-filled workspace for the calls of a shape and says so
    (QSIM_WORKSPACE_KEPT): no clearing launch, and call after call on new data, with either
    rounding, in place or not, aligned or one element off (which takes another single-pass form on
    the same workspace), stays exact; no workgroup ever gives up waiting on the idle GPU."""
    outer, nblocks, inner = shape
    n = outer * nblocks * inner
    ws = torch.zeros(Q.block_workspace_bytes(n, outer, nblocks, inner), dtype=torch.uint8, device="cuda")
    pad = torch.zeros(n + 8, device="cuda")
    for call, (seed, mode, off, in_place) in enumerate([(1, RN_EVEN, 0, False), (2, STOCHASTIC, 0, True), (3, STOCHASTIC, 1, False),
                                                        (4, RN_EVEN, 0, False), (5, STOCHASTIC, 3, True), (6, STOCHASTIC, 0, False)]):
        x = W.lognormal_gradients((n,), seed=seed)
        x[(seed * 7919) % n] = np.float32(3.0e5 * seed)             # the block maximum moves from call to call
        want = R.block_quantize(x, outer, nblocks, inner, 8, mode, 0, 77, call)
        view = pad[off:off + n]
        view.copy_(torch.from_numpy(x))
        out = view if in_place else torch.empty_like(view)
        Q.block_quantize(view, outer, nblocks, inner, 8, mode, Q.WORKSPACE_KEPT, 77, call, out=out, workspace=ws)
        assert_bit_equal(host(out), want, f"{shape} call {call}")
    assert Q.workspace_timeouts(ws) == 0


@pytest.mark.parametrize("shape", KEPT_SHAPES[:5])
def test_block_kept_workspace_survives_waits_that_run_out(shape):
    """With the wait forced to zero the workgroups help themselves (and are counted); the kept
    workspace is as usable afterwards as before."""
    outer, nblocks, inner = shape
    n = outer * nblocks * inner
    ws = torch.zeros(Q.block_workspace_bytes(n, outer, nblocks, inner), dtype=torch.uint8, device="cuda")
    x = W.lognormal_gradients((n,), seed=21)
    d = dev(x)
    wants = {mode: R.block_quantize(x, outer, nblocks, inner, 8, mode, 0, 5, 9) for mode in (RN_EVEN, STOCHASTIC)}

    def run(mode):
        return host(Q.block_quantize(d, outer, nblocks, inner, 8, mode, Q.WORKSPACE_KEPT, 5, 9, workspace=ws))

    assert_bit_equal(run(STOCHASTIC), wants[STOCHASTIC], "before")
    assert Q.workspace_timeouts(ws) == 0
    Q.set_barrier_wait_us(0)
    try:
        assert_bit_equal(run(STOCHASTIC), wants[STOCHASTIC], "no waiting, stochastic")
        assert_bit_equal(run(RN_EVEN), wants[RN_EVEN], "no waiting, nearest")
    finally:
        Q.set_barrier_wait_us(2000)
    gave_up = Q.workspace_timeouts(ws)
    assert gave_up > 0
    assert_bit_equal(run(RN_EVEN), wants[RN_EVEN], "after")
    assert_bit_equal(run(STOCHASTIC), wants[STOCHASTIC], "after, stochastic")
    assert Q.workspace_timeouts(ws) == gave_up


def test_block_single_pass_clears_a_workspace_that_is_not_kept():
    """Without the flag the workspace may hold anything: every call clears what it needs first."""
    for shape in KEPT_SHAPES[:5]:
        outer, nblocks, inner = shape
        n = outer * nblocks * inner
        x = W.lognormal_gradients((n,), seed=33)
        want = R.block_quantize(x, outer, nblocks, inner, 8, STOCHASTIC, 0, 1, 2)
        d = dev(x)
        ws = torch.full((Q.block_workspace_bytes(n, outer, nblocks, inner),), 0xFF, dtype=torch.uint8, device="cuda")
        for fill in (0xFF, 0x80, 0x01):
            ws.fill_(fill)
            assert_bit_equal(host(Q.block_quantize(d, outer, nblocks, inner, 8, STOCHASTIC, 0, 1, 2, workspace=ws)), want,
                             f"{shape} workspace filled with {fill:#x}")
        assert Q.workspace_timeouts(ws) == 0


@pytest.mark.parametrize("log2n", [20, 22, 23, 24])
def test_block_single_pass_meets_without_waiting_out(log2n):
    """On an otherwise idle GPU every workgroup of the single-pass kernel gets a slot, so the
    bounded wait never runs out: a call takes microseconds, not the wait limit."""
    n = 1 << log2n
    x = dev(W.row_scaled_matrix(1, n, seed=log2n))
    out = torch.empty_like(x)
    ws = torch.empty(Q.block_workspace_bytes(n, 1, 1, n), dtype=torch.uint8, device="cuda")
    for mode in (RN_EVEN, STOCHASTIC):
        Q.block_quantize(x, 1, 1, n, 8, mode, 0, 1, 0, out=out, workspace=ws)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for k in range(5):
            Q.block_quantize(x, 1, 1, n, 8, mode, 0, 1, k, out=out, workspace=ws)
        b.record()
        torch.cuda.synchronize()
        assert a.elapsed_time(b) / 5 < 1.0, f"n=2^{log2n} mode {mode}: {a.elapsed_time(b) / 5:.3f} ms per call"


def test_block_whole_tensor_beyond_register_capacity():
    """A single block of 20 Mi elements does not fit in the chip's registers: two streaming passes."""
    for n in (5 * (1 << 22), 5 * (1 << 22) + 3):        # the second ends in a partial group
        x = W.row_scaled_matrix(1, n, seed=77)
        _block_case(x, 1, 1, n, 8, STOCHASTIC)


def test_block_workspace_next_to_the_arrays():
    """Scratch that touches the arrays without overlapping them is accepted; overlapping scratch is not."""
    n = 1 << 18
    need = Q.block_workspace_bytes(n, 1, 1, n)
    assert need > 0
    x = W.row_scaled_matrix(1, n, seed=4).reshape(-1)
    pad = (need + 3) // 4
    buf = torch.zeros(2 * n + 2 * pad, device="cuda")
    buf[pad:pad + n] = dev(x)
    inp, out = buf[pad:pad + n], buf[pad + n:pad + 2 * n]
    want = R.block_quantize(x, 1, 1, n, 8, STOCHASTIC, 0, 3, 4)
    for ws in (buf[:pad], buf[pad + 2 * n:]):
        got = Q.block_quantize(inp, 1, 1, n, 8, STOCHASTIC, 0, 3, 4, out=out, workspace=ws.view(torch.uint8))
        assert_bit_equal(host(got), want, "scratch adjacent to the arrays")
    with pytest.raises(Q.QsimError) as e:
        Q.block_quantize(inp, 1, 1, n, 8, STOCHASTIC, 0, 3, 4, out=out, workspace=buf[pad + n - 4:].view(torch.uint8))
    assert e.value.status == 5


def test_block_with_nonfinite_elements():
    x = W.row_scaled_matrix(4, 2048, seed=2)
    x[1, 3] = np.nan
    x[2, 9] = np.inf
    x[2, 10] = -np.inf
    x[3, 0] = -np.inf
    _block_case(x, 1, 4, 2048, 8, RN_EVEN)
    _block_case(x, 1, 1, 4 * 2048, 8, STOCHASTIC)


# One view per kernel form of the block quantizer, named by the kernel it is served by (checked with a
# kernel trace of this test).
BLOCK_FORMS = [
    (1, 96, 1280),            # block_cached_kernel: contiguous rows, several per workgroup, in registers
    (1, 600, 7),              # block_ragged_kernel: contiguous rows of odd length
    (1, 40, 16381),           # block_rows_kernel: odd rows just under 16 Ki elements
    (1, 3, 70001),            # block_cluster_ragged_kernel: long odd rows, single pass block by block
    (1, 1, 3000000),          # block_resident_kernel: whole tensor, single pass over resident workgroups
    (1, 80, 262144),          # block_resident_kernel block by block: more aligned rows than the chip holds
    (64, 96, 3136),           # block_cluster_strided_kernel: per channel, aligned segments
    (40, 64, 3025),           # block_cluster_ragged_kernel: per channel, odd segments
    (32, 128, 1024),          # block_strided_wide_kernel: per channel, one large workgroup per block
    (2, 3000, 64),            # block_strided_packed_kernel: short blocks along an inner dimension
    (2, 3000, 154),           # block_ragged_runs_kernel: the same with odd segments
    (129, 5000, 1),           # block_ragged_runs_kernel with 16 groups per thread
    (300000, 24, 1),          # block_flat_*: short rows, one element per block and row
    (300000, 9, 4),           # block_flat_*: whole groups
    (70000, 13, 11),          # block_flat_*: odd segments
    (129, 70000, 1),          # block_column_*: one column per block
    (600, 9000, 3),           # block_column_*: odd segments, rows of 27,000
    (2, 2, 4194305),          # block_partial_max_kernel + block_apply_kernel: blocks beyond eight million elements
]


@pytest.mark.parametrize("rounding", [RN_EVEN, RN_AWAY, STOCHASTIC])
@pytest.mark.parametrize("shape", BLOCK_FORMS, ids=lambda s: "x".join(map(str, s)))
def test_block_forms_with_finite_and_with_other_blocks(shape, rounding):
    """Every form quantizes a block without Inf and NaN by a shorter sequence than one with them
    (nearest-even additionally needs the block's exponent to leave room for an anchor 2^(q+23)).
    The same tensor four times: all finite; one NaN; one Inf and one -Inf in different blocks; one
    block whose largest magnitude is near the top of fp32."""
    outer, nblocks, inner = shape
    n = outer * nblocks * inner
    base = W.normal_tensor(n, seed=n % 1000 + 17)
    for case in range(4):
        x = base.copy()
        if case == 1:
            x[(2 * n) // 3] = np.nan
        elif case == 2:
            x[n // 5] = np.inf
            x[n - 1 - n // 7] = -np.inf
        elif case == 3:
            x[n // 2] = np.float32(-3.1e38)
            x[n // 2 + 1 if n // 2 + 1 < n else 0] = np.float32(1.7e35)
        for flags in (0, SYMMETRIC):
            _block_case(x, outer, nblocks, inner, 8, rounding, flags=flags, seed=77 + case, stream_id=5)


@pytest.mark.parametrize("wl,rounding,flags", [(8, RN_EVEN, 0), (24, RN_EVEN, SYMMETRIC), (24, RN_EVEN, 0)])
def test_block_every_encoding_below_the_shared_exponent(wl, rounding, flags):
    """Blocks whose shared exponent is 0 (each row ends in +-1.5 and two more values of that binade)
    over every non-negative fp32 encoding below 2.0, and a sample of the negative ones: the
    nearest-even form that rounds by adding and subtracting 2^(q+23), against the oracle.  With 24
    bits and the most negative code allowed, the tail's -1.9999999 ties up to -2.0 = -2^(q+23) itself."""
    rows, cols = 64, 1 << 20
    tail = np.array([1.5, -1.5, 1.0, -1.9999999], dtype=np.float32)
    starts = list(range(0, 0x40000000, rows * cols)) + [0x80000000, 0xB0000000, 0xBC000000]
    for start in starts:
        body = np.arange(start, start + rows * cols, dtype=np.uint64).astype(np.uint32).view(np.float32).reshape(rows, cols)
        x = np.concatenate([body, np.tile(tail, (rows, 1))], axis=1).reshape(-1)
        _block_case(x, 1, rows, cols + 4, wl, rounding, flags=flags)


# ------------------------------------------------------------------------------------------------
# fused SGD step
# ------------------------------------------------------------------------------------------------
def _fmt(mod, kind, a, b, rounding, flags):
    return mod.Format(kind, a, b, rounding, flags)


SGD_FORMATS = [
    # grad, momentum, weight
    ((1, 5, 2, STOCHASTIC, 3), (2, 16, 12, STOCHASTIC, 1), (3, 8, 256, RN_EVEN, 0)),
    ((1, 5, 2, STOCHASTIC, 3), (2, 16, 12, RN_EVEN, 1), (3, 8, 256, STOCHASTIC, 0)),
    ((0, 0, 0, 0, 0), (0, 0, 0, 0, 0), (0, 0, 0, 0, 0)),
    ((2, 8, 10, RN_AWAY, 1), (1, 8, 7, RN_ZERO, 1), (1, 5, 10, STOCHASTIC, 3)),
    ((3, 8, 64, STOCHASTIC, 0), (3, 12, 1024, STOCHASTIC, 0), (3, 6, 4, STOCHASTIC, 4)),
    ((3, 8, 512, RN_EVEN, 0), (3, 8, 128, RN_AWAY, 4), (3, 8, 8, RN_ZERO, 0)),
    ((0, 0, 0, 0, 0), (2, 16, 12, STOCHASTIC, 1), (2, 8, 6, STOCHASTIC, 5)),
    ((1, 4, 3, RN_EVEN, 1), (0, 0, 0, 0, 0), (3, 8, 16, RN_EVEN, 0)),
]


@pytest.mark.parametrize("formats", SGD_FORMATS)
@pytest.mark.parametrize("n", [1024 * 5, 1024 * 3 + 700 + 3, 37, 1])
def test_sgd_step(formats, n):
    w, g, m = W.sgd_state(n)
    lr, mu, seed = 0.1, 0.9, 1234
    wd, gd, md, qd = dev(w), dev(g), dev(m), torch.full((n,), 7.0, device="cuda")
    wr, mr = w, m
    for step in (2, 3):                      # two steps: the second runs on quantized state
        fo = [_fmt(R, *f) for f in formats]
        fq = [_fmt(Q, *f) for f in formats]
        wr, wqr, mr = R.quant_sgd_step(wr, g, mr, lr, mu, fo[0], fo[1], fo[2], seed, step)
        Q.quant_sgd_step(wd, gd, md, lr, mu, fq[0], fq[1], fq[2], seed, step, w_q=qd)
        assert_bit_equal(host(md), mr, f"momentum, step {step}")
        assert_bit_equal(host(wd), wr, f"master weights, step {step}")
        assert_bit_equal(host(qd), wqr, f"quantized weights, step {step}")
    assert_bit_equal(host(gd), g, "gradient is read only")


def test_sgd_without_wq_and_misaligned():
    n = 5000
    w, g, m = W.sgd_state(n + 4)
    f = SGD_FORMATS[0]
    fo = [_fmt(R, *x) for x in f]
    fq = [_fmt(Q, *x) for x in f]
    wr, _, mr = R.quant_sgd_step(w[1:n + 1], g[2:n + 2], m[:n], 0.1, 0.9, fo[0], fo[1], fo[2], 7, 1, want_wq=False)
    wd, gd, md = dev(w), dev(g), dev(m)
    Q.quant_sgd_step(wd[1:n + 1], gd[2:n + 2], md[:n], 0.1, 0.9, fq[0], fq[1], fq[2], 7, 1)
    assert_bit_equal(host(wd)[1:n + 1], wr, "w")
    assert_bit_equal(host(md)[:n], mr, "mom")
    assert_bit_equal(host(wd)[[0, n + 1, n + 2, n + 3]], w[[0, n + 1, n + 2, n + 3]], "outside w")
    assert_bit_equal(host(md)[n:], m[n:], "outside mom")


@pytest.mark.parametrize("wd,damp,nesterov", [(5e-4, 0.0, 0), (0.0, 0.25, 0), (0.0, 0.0, 1), (1e-2, 0.5, 1)])
@pytest.mark.parametrize("formats", [SGD_FORMATS[0], SGD_FORMATS[2], SGD_FORMATS[4]])
def test_sgd_options(formats, wd, damp, nesterov):
    """Weight decay, dampening and Nesterov momentum, single tensor and multi-tensor."""
    n = 1024 * 3 + 333
    w, g, m = W.sgd_state(n)
    fo = [_fmt(R, *f) for f in formats]
    fq = [_fmt(Q, *f) for f in formats]
    wr, wqr, mr = R.quant_sgd_step(w, g, m, 0.1, 0.9, fo[0], fo[1], fo[2], 1234, 6, options=R.SgdOptions(wd, damp, nesterov))
    wd_, gd, md, qd = dev(w), dev(g), dev(m), torch.empty(n, device="cuda")
    Q.quant_sgd_step(wd_, gd, md, 0.1, 0.9, fq[0], fq[1], fq[2], 1234, 6, w_q=qd, options=Q.SgdOptions(wd, damp, nesterov))
    assert_bit_equal(host(md), mr, "momentum")
    assert_bit_equal(host(wd_), wr, "weights")
    assert_bit_equal(host(qd), wqr, "quantized weights")
    # the same tensor as entry 1 of a list: stream 5 + 1
    w2, g2, m2 = [dev(w[:100]), dev(w)], [dev(g[:100]), dev(g)], [dev(m[:100]), dev(m)]
    Q.quant_sgd_step_multi(w2, g2, m2, 0.1, 0.9, fq[0], fq[1], fq[2], 1234, 5, options=Q.SgdOptions(wd, damp, nesterov))
    assert_bit_equal(host(w2[1]), wr, "weights through the multi-tensor call")
    assert_bit_equal(host(m2[1]), mr, "momentum through the multi-tensor call")
    # and through the device table, every tensor aligned, several steps on one table
    w3, g3, m3 = [dev(w[:100]), dev(w)], [dev(g[:100]), dev(g)], [dev(m[:100]), dev(m)]
    lst = Q.SgdTensorList(w3, g3, m3)
    lst.step(0.1, 0.9, fq[0], fq[1], fq[2], 1234, 5, options=Q.SgdOptions(wd, damp, nesterov))
    assert_bit_equal(host(w3[1]), wr, "weights through the table")
    assert_bit_equal(host(m3[1]), mr, "momentum through the table")
    wr2, _, mr2 = R.quant_sgd_step(wr, g, mr, 0.1, 0.9, fo[0], fo[1], fo[2], 1234, 8, options=R.SgdOptions(wd, damp, nesterov))
    lst.step(0.1, 0.9, fq[0], fq[1], fq[2], 1234, 7, options=Q.SgdOptions(wd, damp, nesterov))
    assert_bit_equal(host(w3[1]), wr2, "weights after a second step on the same table")
    assert_bit_equal(host(m3[1]), mr2, "momentum after a second step on the same table")


def test_sgd_weights_kept_in_the_weight_format():
    n = 1024 * 4 + 99
    w, g, m = W.sgd_state(n)
    f = SGD_FORMATS[0]
    fo = [_fmt(R, *x) for x in f]
    fq = [_fmt(Q, *x) for x in f]
    wr, _, mr = R.quant_sgd_step(w, g, m, 0.1, 0.9, fo[0], fo[1], fo[2], 7, 1, in_place_weights=True)
    wd, gd, md = dev(w), dev(g), dev(m)
    Q.quant_sgd_step(wd, gd, md, 0.1, 0.9, fq[0], fq[1], fq[2], 7, 1, w_q=wd)
    assert_bit_equal(host(wd), wr, "weights stored in the weight format")
    assert_bit_equal(host(md), mr, "momentum")


@pytest.mark.parametrize("entry", ["arrays", "table"])
@pytest.mark.parametrize("formats", [SGD_FORMATS[0], SGD_FORMATS[4], SGD_FORMATS[2]])
def test_sgd_multi_tensor(formats, entry):
    """One call over a model-like list of tensors equals one oracle step per tensor with stream_id + t:
    more than 64 tensors (several launches of the pointer-array entry, one of the device-table entry),
    empty ones, ragged sizes, an unaligned view, missing w_q."""
    def multi(ws, gs, ms, *args, w_q=None, **kw):
        lst = Q.SgdTensorList(ws, gs, ms, w_q)
        (lst.step if entry == "table" else lst.step_batched)(*args, **kw)

    g0 = np.random.Generator(np.random.PCG64(3))
    sizes = [int(v) for v in g0.integers(1, 5000, size=90)] + [0, 64, 1024, 4096, 0, 100000, 3, 147 * 64, 512 * 1024 + 5]
    fo = [_fmt(R, *f) for f in formats]
    fq = [_fmt(Q, *f) for f in formats]
    hw, hg, hm, dw, dg, dm, dq = [], [], [], [], [], [], []
    for t, n in enumerate(sizes):
        w, g, m = W.sgd_state(n + 1, seeds=(100 + t, 200 + t, 300 + t))
        off = 1 if t == 5 else 0                      # one tensor is a misaligned view
        hw.append(w[off:off + n]), hg.append(g[off:off + n]), hm.append(m[off:off + n])
        dw.append(dev(w)[off:off + n]), dg.append(dev(g)[off:off + n]), dm.append(dev(m)[off:off + n])
        dq.append(None if t % 7 == 3 else torch.empty(n, device="cuda"))
    multi(dw, dg, dm, 0.05, 0.9, fq[0], fq[1], fq[2], seed=1234, stream_id=10, w_q=dq)
    for t, n in enumerate(sizes):
        wr, wqr, mr = R.quant_sgd_step(hw[t], hg[t], hm[t], 0.05, 0.9, fo[0], fo[1], fo[2], 1234, 10 + t)
        assert_bit_equal(host(dm[t]), mr, f"momentum of tensor {t} (n={n})")
        assert_bit_equal(host(dw[t]), wr, f"weights of tensor {t} (n={n})")
        if dq[t] is not None:
            assert_bit_equal(host(dq[t]), wqr, f"quantized weights of tensor {t} (n={n})")
    # no quantized copies at all
    dw2 = [dev(x) for x in hw]
    dm2 = [dev(x) for x in hm]
    multi(dw2, dg, dm2, 0.05, 0.9, fq[0], fq[1], fq[2], seed=1234, stream_id=10)
    for t in (0, 17, 40, 63, 64, 90, 95, 98):
        assert_bit_equal(host(dw2[t]), host(dw[t]), f"tensor {t} without w_q")


# ------------------------------------------------------------------------------------------------
# the benchmark's workloads at full size
# ------------------------------------------------------------------------------------------------
def test_full_workload_1_float_e5m2():
    x = W.normal_tensor()
    for flags in (SATURATE, SATURATE | SUBNORMAL):
        want = R.float_quantize(x, 5, 2, RN_EVEN, flags, threads=THREADS)
        assert_bit_equal(host(Q.float_quantize(dev(x), 5, 2, RN_EVEN, flags)), want, f"E5M2 flags {flags}")


def test_full_workload_2_fixed_stochastic():
    x = W.uniform_with_outliers()
    want = R.fixed_quantize(x, 8, 6, STOCHASTIC, SATURATE, seed=1234, threads=THREADS)
    got = host(Q.fixed_quantize(dev(x), 8, 6, STOCHASTIC, SATURATE, seed=1234))
    assert_bit_equal(got, want, "fixed(8,6) stochastic, 64 Mi elements")
    assert 0.45 < float(np.mean((np.abs(x) >= 2.0))) < 0.6          # about half the elements saturate


@pytest.mark.parametrize("rounding", [RN_EVEN, STOCHASTIC])
def test_full_workload_3_block(rounding):
    x = W.row_scaled_matrix()
    _block_case(x, 1, 4096, 4096, 8, rounding, seed=1234, stream_id=0)
    _block_case(x, 1, 1, 4096 * 4096, 8, rounding, seed=1234, stream_id=0)


def test_full_workload_4_activations_and_gradients():
    a = W.relu_activations()
    want = R.float_quantize(a, 8, 7, STOCHASTIC, SATURATE | SUBNORMAL, seed=1234, threads=THREADS)
    assert_bit_equal(host(Q.float_quantize(dev(a), 8, 7, STOCHASTIC, SATURATE | SUBNORMAL, seed=1234)), want, "E8M7 stochastic")
    del a, want
    g = W.lognormal_gradients(overflow_fraction=2.0 ** -10)
    for flags in (SATURATE | SUBNORMAL, 0):
        want = R.float_quantize(g, 5, 10, RN_EVEN, flags, threads=THREADS)
        assert_bit_equal(host(Q.float_quantize(dev(g), 5, 10, RN_EVEN, flags)), want, f"E5M10 flags {flags}")
    sub = np.abs(g) < 2.0 ** -14
    assert 0.2 < float(sub.mean()) < 0.6 and float((np.abs(g) > 65504).mean()) > 0


def test_full_workload_4_block_per_channel():
    """The [128, 256, 56, 56] activation tensor with one shared exponent per channel, as bench.py times it."""
    a = W.relu_activations()
    n, c, hw = a.shape[0], a.shape[1], a.shape[2] * a.shape[3]
    want = R.block_quantize(a, n, c, hw, 8, STOCHASTIC, 0, 1234, 0).reshape(-1)
    got = host(Q.block_quantize(dev(a.reshape(-1)), n, c, hw, 8, STOCHASTIC, 0, 1234, 0))
    assert_bit_equal(got, want, "block8 per channel, stochastic, 102,760,448 elements")


@pytest.mark.parametrize("n", [W.N_PARAMS, W.N_PARAMS_RAGGED])
def test_full_workload_5_sgd(n):
    w, g, m = W.sgd_state(n)
    fmts = SGD_FORMATS[0]
    fo = [_fmt(R, *f) for f in fmts]
    fq = [_fmt(Q, *f) for f in fmts]
    m = R.fixed_quantize(m, 16, 12, STOCHASTIC, SATURATE, seed=8, threads=THREADS)   # start from a quantized momentum
    wr, wqr, mr = R.quant_sgd_step(w, g, m, 0.1, 0.9, fo[0], fo[1], fo[2], 1234, 2)
    wd, gd, md, qd = dev(w), dev(g), dev(m), torch.empty(n, device="cuda")
    Q.quant_sgd_step(wd, gd, md, 0.1, 0.9, fq[0], fq[1], fq[2], 1234, 2, w_q=qd)
    assert_bit_equal(host(md), mr, "momentum")
    assert_bit_equal(host(wd), wr, "master weights")
    assert_bit_equal(host(qd), wqr, "quantized weights")


def test_full_workload_5_sgd_over_a_resnet50_parameter_list():
    """The 161 parameter tensors of a ResNet-50 (25.6 M parameters) in one table step, as bench.py times it."""
    sizes = W.resnet50_parameter_sizes()
    total = sum(sizes)
    w, g, m = W.sgd_state(total)
    fmts = SGD_FORMATS[0]
    fo = [_fmt(R, *f) for f in fmts]
    fq = [_fmt(Q, *f) for f in fmts]
    flat = [dev(w), dev(g), dev(m), torch.empty(total, device="cuda")]
    lists = [list(torch.split(f, sizes)) for f in flat]
    Q.SgdTensorList(lists[0], lists[1], lists[2], lists[3]).step(0.1, 0.9, fq[0], fq[1], fq[2], 1234, 2)
    gw, gm, gq = host(flat[0]), host(flat[2]), host(flat[3])
    lo = 0
    for t, n in enumerate(sizes):
        wr, wqr, mr = R.quant_sgd_step(w[lo:lo + n], g[lo:lo + n], m[lo:lo + n], 0.1, 0.9, fo[0], fo[1], fo[2], 1234, 2 + t)
        assert_bit_equal(gm[lo:lo + n], mr, f"momentum of tensor {t} (n={n})")
        assert_bit_equal(gw[lo:lo + n], wr, f"weights of tensor {t} (n={n})")
        assert_bit_equal(gq[lo:lo + n], wqr, f"quantized weights of tensor {t} (n={n})")
        lo += n


def test_block_single_pass_forms_on_two_streams_at_once():
    """Two calls whose workgroups wait for their block-mates run side by side on two streams, each
    with its own scratch: both must finish with exact results."""
    rows, cols = 300, 70000
    shape = (32, 64, 3136)
    x1 = W.row_scaled_matrix(rows, cols, seed=31).reshape(-1)
    x2 = W.lognormal_gradients(shape, seed=32).reshape(-1)
    want1 = R.block_quantize(x1, 1, rows, cols, 8, STOCHASTIC, 0, 9, 1)
    want2 = R.block_quantize(x2, *shape, 8, STOCHASTIC, 0, 9, 2)
    d1, d2 = dev(x1), dev(x2)
    o1, o2 = torch.empty_like(d1), torch.empty_like(d2)
    ws1 = torch.empty(Q.block_workspace_bytes(d1.numel(), 1, rows, cols), dtype=torch.uint8, device="cuda")
    ws2 = torch.empty(Q.block_workspace_bytes(d2.numel(), *shape), dtype=torch.uint8, device="cuda")
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(5):
        with torch.cuda.stream(s1):
            Q.block_quantize(d1, 1, rows, cols, 8, STOCHASTIC, 0, 9, 1, out=o1, workspace=ws1)
        with torch.cuda.stream(s2):
            Q.block_quantize(d2, *shape, 8, STOCHASTIC, 0, 9, 2, out=o2, workspace=ws2)
    torch.cuda.synchronize()
    assert_bit_equal(host(o1), want1, "rows, stream 1")
    assert_bit_equal(host(o2), want2, "channels, stream 2")
