"""Developer scans of block floating point over shapes: which kernel form serves which shape, and
how well.  Not part of the library's surface; kept because the summaries under profiles/ name these
commands.  Every call leaves the scratch to the binding, which keeps a zero-filled one per shape
(QSIM_WORKSPACE_KEPT), as a training loop that calls the same shapes every step would.

    python -m paper_1910_04540_amd.tuning_scans --block-shapes

times block floating point with one block per row over row lengths from 1 to the whole tensor
(64 Mi elements in all, three rotating buffer sets).

    python -m paper_1910_04540_amd.tuning_scans --shape-scan SEED

times some 200 seeded random views [outer, nblocks, inner] of a tensor of up to 32 Mi elements
(sizes spread over orders of magnitude, half of the inner lengths rounded to multiples of four) and
prints the slowest shapes and the quartiles: a search for shapes that no kernel form serves well.

    python -m paper_1910_04540_amd.tuning_scans --channel-shapes

times one block per channel (arXiv 1910.04540, Sec. 3.1: a block over an arbitrary dimension) over
activation tensors [N, C, H, W] of the shapes convolutional networks produce: the paper's VGG-16 on
32 x 32 images, and ImageNet-sized networks with spatial sizes that are (56 x 56, 28 x 28) and are
not (55 x 55, 27 x 27, 35 x 35) multiples of four elements.
"""
from __future__ import annotations

import argparse
import sys

import torch

from . import binding as Q
from .sweep import _time

BLOCK_ROW_LENGTHS = [1, 3, 4, 10, 16, 27, 64, 100, 256, 1000, 1001, 1024, 4096, 4098, 16384, 16388, 25088, 29799, 65536,
                     1000003, 1 << 20, 1 << 24, 1 << 26]


def block_shapes() -> int:
    """Per-row block quantize of 64 Mi elements for a range of row lengths."""
    total = 1 << 26
    xs = [torch.randn(total, device="cuda") for _ in range(3)]
    outs = [torch.empty(total, device="cuda") for _ in range(3)]
    print(f"{'rows':>10} {'row length':>10} | {'nearest us':>10} {'% of 8 TB/s':>11} | {'stochastic us':>13} {'% of 8 TB/s':>11}")
    for cols in BLOCK_ROW_LENGTHS:
        rows = total // cols
        n = rows * cols
        cells = []
        for mode in (Q.RN_EVEN, Q.STOCHASTIC):
            turn = [0]

            def call():
                k = turn[0] % 3
                turn[0] += 1
                Q.block_quantize(xs[k][:n], 1, rows, cols, 8, mode, 0, 1, 0, out=outs[k][:n])

            for _ in range(100):
                call()
            us = _time(call, 100)
            cells.append((us, n * 8 / us / 1e3 / 80.0))
        print(f"{rows:>10} {cols:>10} | {cells[0][0]:10.1f} {cells[0][1]:11.1f} | {cells[1][0]:13.1f} {cells[1][1]:11.1f}", flush=True)
    return 0


CHANNEL_SHAPES = [
    # VGG-16 on CIFAR-10 images, batch 128 (Sec. 5)
    (128, 64, 32, 32), (128, 128, 16, 16), (128, 256, 8, 8), (128, 512, 4, 4), (128, 512, 2, 2),
    # ImageNet-sized feature maps, whole groups per row of the view
    (128, 64, 112, 112), (128, 256, 56, 56), (128, 512, 28, 28), (128, 1024, 14, 14), (128, 2048, 7, 7),
    # the same with odd spatial sizes
    (128, 64, 55, 55), (128, 192, 27, 27), (128, 384, 13, 13), (64, 288, 35, 35), (64, 768, 17, 17), (32, 3, 299, 299),
]


def channel_shapes() -> int:
    """Per-channel block quantize of [N, C, H, W] activations: the view [N, C, H * W], one block per C."""
    print(f"{'N, C, H, W':>20} {'elements':>10} | {'nearest us':>10} {'% of 8 TB/s':>11} | {'stochastic us':>13} {'% of 8 TB/s':>11}")
    for shape in CHANNEL_SHAPES:
        batch, channels, height, width = shape
        inner = height * width
        n = batch * channels * inner
        xs = [torch.randn(n, device="cuda") for _ in range(3)]
        out = torch.empty(n, device="cuda")
        cells = []
        for mode in (Q.RN_EVEN, Q.STOCHASTIC):
            turn = [0]

            def call():
                turn[0] += 1
                Q.block_quantize(xs[turn[0] % 3], batch, channels, inner, 8, mode, 0, 1, 0, out=out)

            for _ in range(30):
                call()
            us = _time(call, 50)
            cells.append((us, n * 8 / us / 1e3 / 80.0))
        label = ", ".join(str(v) for v in shape)
        print(f"{label:>20} {n:>10} | {cells[0][0]:10.1f} {cells[0][1]:11.1f} | {cells[1][0]:13.1f} {cells[1][1]:11.1f}", flush=True)
        del xs, out
        torch.cuda.empty_cache()
    return 0


def shape_scan(seed: int) -> int:
    import numpy as np

    g = np.random.Generator(np.random.PCG64(seed))
    total = 1 << 25
    x = torch.randn(total + 64, device="cuda")
    out = torch.empty(total + 64, device="cuda")
    rows = []
    for _ in range(220):
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
        if n > total or n < total // 4:
            continue
        need = Q.block_workspace_bytes(n, outer, nblocks, inner)
        if need > (1 << 31):
            continue
        for mode, name in ((Q.RN_EVEN, "nearest"), (Q.STOCHASTIC, "stochastic")):
            call = lambda: Q.block_quantize(x[:n], outer, nblocks, inner, 8, mode, 0, 1, 0, out=out[:n])
            for _ in range(4):
                call()
            us = min(_time(call, 8), _time(call, 8))      # (the better of two: a hiccup of the host shows in eight calls)
            rows.append((n * 8 / us / 1e3 / 80.0, us, outer, nblocks, inner, n, name))
    rows.sort()
    print(f"{len(rows)} timings (shape x rounding), % of 8 TB/s at 8 B per element; slowest first")
    for r in rows[:12]:
        print(f"{r[0]:5.1f} %  {r[1]:8.1f} us  [{r[2]}, {r[3]}, {r[4]}]  n={r[5]}  {r[6]}")
    q = [rows[int(len(rows) * f)][0] for f in (0.0, 0.25, 0.5, 0.75)] + [rows[-1][0]]
    print("minimum, quartiles, maximum: " + ", ".join(f"{v:.1f} %" for v in q))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--block-shapes", action="store_true")
    ap.add_argument("--channel-shapes", action="store_true")
    ap.add_argument("--shape-scan", type=int, default=None, metavar="SEED")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("the scans need a GPU", file=sys.stderr)
        return 2
    Q.lib()
    if args.block_shapes:
        return block_shapes()
    if args.channel_shapes:
        return channel_shapes()
    if args.shape_scan is not None:
        return shape_scan(args.shape_scan)
    ap.print_help()
    return 2


if __name__ == "__main__":
    sys.exit(main())
