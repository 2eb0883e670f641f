"""The entry points allocate nothing and never synchronise, so a sequence of calls can be captured
in a HIP graph and replayed; every replay must give what eager calls give on the same inputs."""
import numpy as np
import pytest

from helpers import assert_bit_equal

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from paper_1910_04540_amd import binding as Q       # noqa: E402
from paper_1910_04540_amd import workloads as W     # noqa: E402


def test_graph_replays_match_eager_calls():
    if not torch.cuda.is_available():
        pytest.fail("needs a GPU")
    n, rows, cols = 50000, 24, 4096
    nw = 1 << 18
    x = torch.empty(n, device="cuda")
    mat = torch.empty(rows * cols, device="cuda")
    whole = torch.empty(nw, device="cuda")
    w, g, m = (torch.empty(n, device="cuda") for _ in range(3))
    out = {k: torch.empty_like(v) for k, v in (("fixed", x), ("float", x), ("rows", mat), ("whole", whole))}
    wq = torch.empty(n, device="cuda")
    ws = torch.empty(Q.block_workspace_bytes(nw, 1, 1, nw), dtype=torch.uint8, device="cuda")
    fg, fm, fw = Q.Format(1, 5, 2, 3, 3), Q.Format(2, 16, 12, 3, 1), Q.Format(3, 8, 256, 0, 0)

    def calls(o, wt, mt, wqt):
        Q.fixed_quantize(x, 8, 6, Q.STOCHASTIC, Q.SATURATE, 1234, 1, out=o["fixed"])
        Q.float_quantize(x, 5, 2, Q.RN_EVEN, Q.SATURATE | Q.SUBNORMAL, out=o["float"])
        Q.block_quantize(mat, 1, rows, cols, 8, Q.STOCHASTIC, 0, 7, 2, out=o["rows"])
        Q.block_quantize(whole, 1, 1, nw, 8, Q.STOCHASTIC, 0, 7, 3, out=o["whole"], workspace=ws)
        Q.quant_sgd_step(wt, g, mt, 0.1, 0.9, fg, fm, fw, 99, 4, w_q=wqt)

    def fill(seed):
        x.copy_(torch.from_numpy(W.uniform_with_outliers(n, seed=seed)))
        mat.copy_(torch.from_numpy(W.row_scaled_matrix(rows, cols, seed=seed + 1).reshape(-1)))
        whole.copy_(torch.from_numpy(W.row_scaled_matrix(1, nw, seed=seed + 2).reshape(-1)))
        a, b, c = W.sgd_state(n, seeds=(seed + 3, seed + 4, seed + 5))
        w.copy_(torch.from_numpy(a)), g.copy_(torch.from_numpy(b)), m.copy_(torch.from_numpy(c))

    fill(1)
    calls(out, w.clone(), m.clone(), wq)            # warm-up outside the capture (first-use queries happen here)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        calls(out, w, m, wq)
    for replay in range(3):
        fill(10 * replay + 20)
        w0, m0 = w.clone(), m.clone()
        eager = {k: torch.empty_like(v) for k, v in out.items()}
        ew, em, ewq = w0.clone(), m0.clone(), torch.empty_like(wq)
        calls(eager, ew, em, ewq)                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in out:
            assert_bit_equal(out[k].cpu().numpy(), eager[k].cpu().numpy(), f"{k}, replay {replay}")
        assert_bit_equal(w.cpu().numpy(), ew.cpu().numpy(), f"weights, replay {replay}")
        assert_bit_equal(m.cpu().numpy(), em.cpu().numpy(), f"momentum, replay {replay}")
        assert_bit_equal(wq.cpu().numpy(), ewq.cpu().numpy(), f"quantized weights, replay {replay}")


def test_graph_replays_the_table_step():
    """The device-table step is one kernel launch, so it can be captured once its table is built
    (building copies from the host and waits, which a capture cannot hold)."""
    if not torch.cuda.is_available():
        pytest.fail("needs a GPU")
    sizes = [5000, 1, 0, 1024, 70001, 333]
    total = sum(sizes)
    w, g, m = (torch.empty(total, device="cuda") for _ in range(3))
    fg, fm, fw = Q.Format(1, 5, 2, 3, 3), Q.Format(2, 16, 12, 3, 1), Q.Format(3, 8, 256, 0, 0)
    split = lambda t: list(torch.split(t, sizes))
    captured = Q.SgdTensorList(split(w), split(g), split(m))

    def fill(seed):
        a, b, c = W.sgd_state(total, seeds=(seed, seed + 1, seed + 2))
        w.copy_(torch.from_numpy(a)), g.copy_(torch.from_numpy(b)), m.copy_(torch.from_numpy(c))

    fill(1)
    captured.step(0.1, 0.9, fg, fm, fw, 5, 9)       # builds the table
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        captured.step(0.1, 0.9, fg, fm, fw, 5, 9)
    for replay in range(3):
        fill(50 + 3 * replay)
        ew, em = w.clone(), m.clone()
        Q.SgdTensorList(split(ew), split(g), split(em)).step_batched(0.1, 0.9, fg, fm, fw, 5, 9)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_bit_equal(w.cpu().numpy(), ew.cpu().numpy(), f"weights, replay {replay}")
        assert_bit_equal(m.cpu().numpy(), em.cpu().numpy(), f"momentum, replay {replay}")


def test_graph_replays_every_block_form():
    """Every multi-launch block form (single pass block by block over aligned and over odd segments,
    packed, flat, column, two-pass, the split max / quantize pair) captured once and replayed on new data."""
    if not torch.cuda.is_available():
        pytest.fail("needs a GPU")
    shapes = [(32, 64, 3136), (2, 3000, 64), (5000, 3, 300), (300, 4096, 1), (9, 6, 20714), (1, 300, 70000), (1, 700, 1001),
              (1, 1, 3 * (1 << 20) + 1), (2, 2, (1 << 21) + 1), (1, 40, 29799)]
    xs = [torch.empty(o * b * i, device="cuda") for o, b, i in shapes]
    outs = [torch.empty_like(x) for x in xs]
    wss = [torch.empty(max(Q.block_workspace_bytes(x.numel(), *s), 16), dtype=torch.uint8, device="cuda") for x, s in zip(xs, shapes)]
    maxima = torch.empty(shapes[0][1], dtype=torch.int32, device="cuda")
    split_out = torch.empty_like(xs[0])

    def calls(dst, dst_split):
        for x, s, o, ws in zip(xs, shapes, dst, wss):
            Q.block_quantize(x, *s, 8, Q.STOCHASTIC, 0, 3, 1, out=o, workspace=ws)
        Q.block_max(xs[0], *shapes[0], out=maxima, workspace=wss[0])
        Q.block_quantize_with_max(xs[0], *shapes[0], 8, maxima, Q.STOCHASTIC, 0, 3, 1, out=dst_split)

    def fill(seed):
        g = np.random.Generator(np.random.PCG64(seed))
        for x in xs:
            x.copy_(torch.from_numpy((g.standard_normal(x.numel(), dtype=np.float32) *
                                      np.exp2(g.integers(-8, 8, x.numel()))).astype(np.float32)))

    fill(1)
    calls(outs, split_out)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        calls(outs, split_out)
    for replay in range(3):
        fill(100 + replay)
        eager = [torch.empty_like(x) for x in xs]
        eager_split = torch.empty_like(xs[0])
        calls(eager, eager_split)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for s, a, b in zip(shapes, outs, eager):
            assert_bit_equal(a.cpu().numpy(), b.cpu().numpy(), f"{s}, replay {replay}")
        assert_bit_equal(split_out.cpu().numpy(), eager_split.cpu().numpy(), f"split pair, replay {replay}")
        assert_bit_equal(split_out.cpu().numpy(), outs[0].cpu().numpy(), f"split pair equals the fused call, replay {replay}")
