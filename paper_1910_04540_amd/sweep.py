"""Wall-clock sweep over tensor sizes: the fused kernels against the "many-kernel" approach.

arXiv 1910.04540, Sec. 4 ("Validation") compares its fused kernels with the same quantization
written as a chain of stock PyTorch operations, one kernel launch each (`many-fixed`,
`many-block`), over a range of tensor sizes, for nearest and stochastic rounding.  This script
repeats that comparison on this GPU: the comparator below is stock torch-ROCm elementwise and
reduction ops; floating point has no such comparator (it needs bit operations), so it is timed alone.

    python -m paper_1910_04540_amd.sweep [--min-log2 10] [--max-log2 28] [--json]

Prints one row per (format, rounding, size): microseconds per call for both approaches and their
ratio.  Nearest rounding of the comparator is checked against the fused result on every size.
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

from . import binding as Q
from . import workloads as W

def many_fixed(x, wl, fl, stochastic):
    """Fixed point (wl, fl), saturating, from stock ops: 4 launches nearest-even, 6 stochastic."""
    y = x * float(2.0 ** fl)
    y = torch.floor(y + torch.rand_like(y)) if stochastic else torch.round(y)
    y = torch.clamp(y, -float(2 ** (wl - 1)), float(2 ** (wl - 1) - 1))
    return y * float(2.0 ** -fl)


def many_block(x, wl, stochastic):
    """Block floating point over the whole tensor from stock ops (the exponent through log2/floor,
    as bit operations are not used): about 10 launches."""
    amax = x.abs().max()
    e = torch.floor(torch.log2(amax))
    step = torch.exp2(e + float(2 - wl))
    y = x / step
    y = torch.floor(y + torch.rand_like(y)) if stochastic else torch.round(y)
    y = torch.clamp(y, -float(2 ** (wl - 1)), float(2 ** (wl - 1) - 1))
    return y * step


def _time(fn, reps):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / reps


def size_sweep(min_log2: int = 10, max_log2: int = 28, step: int = 2, reps: int | None = None) -> list[dict]:
    """One row per (size, rounding): microseconds per call of the fused kernels and of the stock-op
    chains.  On every size the comparator's nearest rounding must reproduce the fused result."""
    rows = []
    base = torch.from_numpy(W.normal_tensor(1 << 20, seed=21)).cuda()
    for lg in range(min_log2, max_log2 + 1, step):
        n = 1 << lg
        x = base.repeat((n + base.numel() - 1) // base.numel())[:n].contiguous()
        out = torch.empty_like(x)
        ws = torch.empty(max(Q.block_workspace_bytes(n, 1, 1, n), 16), dtype=torch.uint8, device="cuda")
        r = reps if reps is not None else (200 if lg <= 20 else (50 if lg <= 24 else 10))
        # nearest rounding: the comparator must agree with the fused kernels
        assert torch.equal(many_fixed(x, 8, 6, False), Q.fixed_quantize(x, 8, 6, Q.RN_EVEN, Q.SATURATE))
        assert torch.equal(many_block(x, 8, False), Q.block_quantize(x, 1, 1, n, 8, Q.RN_EVEN, workspace=ws))
        for sto, name in ((False, "nearest"), (True, "stochastic")):
            mode = Q.STOCHASTIC if sto else Q.RN_EVEN
            fused_fixed = _time(lambda: Q.fixed_quantize(x, 8, 6, mode, Q.SATURATE, 1, 0, out=out), r)
            many_fx = _time(lambda: many_fixed(x, 8, 6, sto), r)
            fused_block = _time(lambda: Q.block_quantize(x, 1, 1, n, 8, mode, 0, 1, 0, out=out, workspace=ws), r)
            many_bl = _time(lambda: many_block(x, 8, sto), r)
            fused_float = _time(lambda: Q.float_quantize(x, 5, 2, mode, Q.SATURATE, 1, 0, out=out), r)
            rows.append({"log2_n": lg, "rounding": name, "fixed_fused_us": fused_fixed, "fixed_many_us": many_fx,
                         "fixed_ratio": many_fx / fused_fixed, "block_fused_us": fused_block, "block_many_us": many_bl,
                         "block_ratio": many_bl / fused_block, "float_fused_us": fused_float})
        del x, out
        torch.cuda.empty_cache()
    return rows


def format_rows(rows: list[dict]) -> str:
    lines = [f"{'n':>6} {'rounding':>10} | {'fixed fused':>11} {'many':>9} {'ratio':>6} | {'block fused':>11} {'many':>9} {'ratio':>6} | "
             f"{'float fused':>11}   (us per call)"]
    for r in rows:
        lines.append(f"2^{r['log2_n']:<4d} {r['rounding']:>10} | {r['fixed_fused_us']:11.1f} {r['fixed_many_us']:9.1f} {r['fixed_ratio']:6.1f} | "
                     f"{r['block_fused_us']:11.1f} {r['block_many_us']:9.1f} {r['block_ratio']:6.1f} | {r['float_fused_us']:11.1f}")
    return "\n".join(lines)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--min-log2", type=int, default=10)
    ap.add_argument("--max-log2", type=int, default=28)
    ap.add_argument("--json", action="store_true")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("the sweep needs a GPU", file=sys.stderr)
        return 2
    Q.lib()
    rows = size_sweep(args.min_log2, args.max_log2)
    if args.json:
        for r in rows:
            print(json.dumps(r))
    else:
        print(format_rows(rows))
    return 0


if __name__ == "__main__":
    sys.exit(main())
