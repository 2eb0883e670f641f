#!/usr/bin/env python3
"""Throughput of the fused quantize-and-round kernels on one MI355X.

A step is one fixed-point quantize call (wl = 8, fl = 6, stochastic rounding, clamp on overflow)
over a 64 Mi-element fp32 tensor that is already resident in HBM.  Inputs rotate over three
buffer sets so that no step finds its tensor in the memory-side cache.  One JSON line is printed:
the headline elements/s, the HBM roofline of the dominant kernel measured with HIP events on
the launch stream, the same figures for the other formats (`formats`), and the CPU oracle timed on
the host cores as a reported baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-formats] [--no-cpu]

Before the W warm-up steps the headline kernel is launched RAMP more times, untimed, so that a run
with a short warm-up does not time the clocks coming up after an idle phase; every row of `formats`
times at least 200 launches after at least 100 warm-up launches of its own.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
BYTES_PER_ELEMENT = 8          # one fp32 read + one fp32 write
SGD_BYTES_PER_PARAM = 24       # three reads + three writes
NSETS = 3

RAMP = 300                     # untimed launches ahead of the warm-up (about 25 ms)

# HBM traffic per launch of the headline kernel, measured with rocprofv3 --pmc (FETCH_SIZE, then
# WRITE_SIZE, each scaled by what the same counter reads for the device-to-device copy below):
# read from the summary of those runs, so that the figure and its evidence cannot drift apart.
TRAFFIC_SUMMARY = os.path.join("profiles", "fixed_sr_64Mi_hbm_counters.txt")


def _measured_traffic():
    """Bytes per launch from the line 'Scaled traffic ... = N bytes' of the summary (None when it is missing)."""
    import re
    try:
        with open(os.path.join(ROOT, TRAFFIC_SUMMARY)) as fh:
            m = re.search(r"Scaled traffic of the qsim kernel per launch:.*=\s*(\d+) bytes", fh.read())
        return int(m.group(1)) if m else None
    except OSError:
        return None


def _time_launches(fn, steps, warmup, torch):
    """fn(k) enqueues launch k on torch's current stream.  Returns (wall seconds, event seconds).

    The device is idle when the host clock starts (torch.cuda.synchronize() just returned, the start
    event is on an empty stream) and the clock stops when the event behind the last launch has been
    reached, found by polling; the synchronize that closes the bracket follows at once and finds the
    device idle.  (On this machine a synchronize of an idle device takes 30-40 us of host time by
    itself, which over 20 steps of 80 us would read as 2 % less throughput than the device delivered.)"""
    for k in range(warmup):
        fn(k)
    torch.cuda.synchronize()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    t0 = time.perf_counter()
    for k in range(steps):
        fn(k)
    stop.record()
    while not stop.query():
        pass
    wall = time.perf_counter() - t0
    torch.cuda.synchronize()
    return wall, start.elapsed_time(stop) * 1e-3


def _rotating(x_host, torch):
    """Three device copies of a workload (rolled so they differ) plus three output buffers."""
    base = torch.from_numpy(x_host).cuda().reshape(-1)
    ins = [base] + [torch.roll(base, 1234567 * (k + 1)) for k in range(NSETS - 1)]
    outs = [torch.empty_like(base) for _ in range(NSETS)]
    return ins, outs


def _entry(name, elements, bytes_per_element, seconds, launches, extra=None):
    per = seconds / launches
    gbs = elements * bytes_per_element / per / 1e9
    d = {"elements": elements, "us_per_call": per * 1e6, "elements_per_s": elements / per, "GBps": gbs,
         "frac_of_hbm_peak": gbs / HBM_PEAK_GBS, "launches_timed": launches}
    if extra:
        d.update(extra)
    return name, d


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=500, help="untimed launches; enough to bring the clocks up after an idle phase")
    ap.add_argument("--no-formats", action="store_true", help="skip the per-format table")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1910_04540_amd import binding as Q
    from paper_1910_04540_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    if not os.path.exists(Q.LIB_PATH):          # load what is built; build only when nothing is
        from paper_1910_04540_amd import build as hip_build
        hip_build.build()
    Q.lib()
    torch.cuda.set_device(0)

    # ---- headline: fixed point (8, 6), stochastic, saturating, 64 Mi elements -----------------
    x_host = W.uniform_with_outliers()
    n = x_host.size
    ins, outs = _rotating(x_host, torch)

    def fixed_step(k):
        Q.fixed_quantize(ins[k % NSETS], 8, 6, Q.STOCHASTIC, Q.SATURATE, seed=1234, stream_id=k, out=outs[k % NSETS])

    for k in range(RAMP):
        fixed_step(k)
    wall, ev = _time_launches(fixed_step, args.steps, args.warmup, torch)
    # a plain device-to-device copy of the same tensor: the known-size reference that scales the
    # profiler's HBM byte counters (it is outside every timed region)
    for k in range(NSETS):
        outs[k].copy_(ins[k])
    torch.cuda.synchronize()
    value = n * args.steps / wall
    achieved = n * BYTES_PER_ELEMENT / (ev / args.steps) / 1e9
    result = {
        "metric": "quantized elements/sec, fixed-point (wl=8, fl=6) stochastic rounding with clamp, 1 MI355X",
        "value": value,
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "fixed_point_quantize 64Mi fp32 (90% U[-4,4) + 10% N(0,sd 10)), wl=8 fl=6, "
                               "stochastic (Philox seed 1234), saturate", "elements": n,
                   "buffer_sets": NSETS, "in_place": False, "clock_ramp_launches": RAMP},
        # `frac` is on the HIP-event clock (the kernel's launches alone); `frac_wall` is the same bytes
        # over the host's clock, which is what `value` and `ms_per_step` are on
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": _measured_traffic(), "traffic_source": TRAFFIC_SUMMARY,
                     "kernel": "qsim::elementwise_kernel<qsim::FixedOp, 3, 1>", "algorithmic_bytes": n * BYTES_PER_ELEMENT,
                     "avg_launch_us": ev / args.steps * 1e6, "avg_launch_us_wall": wall / args.steps * 1e6,
                     "frac_wall": n * BYTES_PER_ELEMENT / (wall / args.steps) / 1e9 / HBM_PEAK_GBS},
    }

    # ---- the other formats ---------------------------------------------------------------------
    if not args.no_formats:
        formats = {}
        reps = max(200, args.steps // 4)
        warm = max(100, args.warmup // 2)

        def run(name, fn, elements, bpe=BYTES_PER_ELEMENT, extra=None, kernel=None, launches=reps):
            """Times `launches` calls of fn after `warm` untimed ones; `kernel`: the kernel(s) of one call,
            named as rocprofv3 prints them, so that the row can be found in profiles/."""
            _, e = _time_launches(fn, launches, warm, torch)
            k, d = _entry(name, elements, bpe, e, launches, extra)
            if kernel:
                d["kernel"] = kernel
            formats[k] = d
            return d

        run("fixed_8_6_nearest_even", lambda k: Q.fixed_quantize(ins[k % NSETS], 8, 6, Q.RN_EVEN, Q.SATURATE,
                                                                   out=outs[k % NSETS]), n,
            kernel="qsim::elementwise_kernel<qsim::FixedOp, 0, 1>")
        run("fixed_8_6_stochastic_in_place", lambda k: Q.fixed_quantize(outs[k % NSETS], 8, 6, Q.STOCHASTIC, Q.SATURATE,
                                                                          seed=1234, stream_id=k, out=outs[k % NSETS]), n,
            extra={"note": "input already quantized by the previous runs"}, kernel="qsim::elementwise_kernel<qsim::FixedOp, 3, 1>")
        del ins, outs
        torch.cuda.empty_cache()

        small = torch.from_numpy(W.normal_tensor()).cuda()
        small_out = torch.empty_like(small)
        run("float_e5m2_nearest_even_1Mi", lambda k: Q.float_quantize(small, 5, 2, Q.RN_EVEN, Q.SATURATE, out=small_out),
            small.numel(), extra={"note": "launch-latency bound, cache resident"},
            kernel="qsim::elementwise_kernel<qsim::FloatShiftOp<false>, 0, 1>")

        # the same small call captured 16 times in a HIP graph: what remains when launch overhead is amortised
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(16):
                Q.float_quantize(small, 5, 2, Q.RN_EVEN, Q.SATURATE, out=small_out)
        _, e = _time_launches(lambda k: graph.replay(), max(10, reps // 4), 10, torch)
        name, d = _entry("float_e5m2_nearest_even_1Mi_in_a_graph_of_16", small.numel(), BYTES_PER_ELEMENT, e,
                         max(10, reps // 4) * 16, {"note": "per call, graph replay; cache resident"})
        d["kernel"] = "qsim::elementwise_kernel<qsim::FloatShiftOp<false>, 0, 1>"
        formats[name] = d
        del graph

        a_in, a_out = _rotating(W.relu_activations().reshape(-1), torch)
        na = a_in[0].numel()
        run("float_e8m7_stochastic_activations", lambda k: Q.float_quantize(
            a_in[k % NSETS], 8, 7, Q.STOCHASTIC, Q.SATURATE | Q.SUBNORMAL, seed=1234, stream_id=k, out=a_out[k % NSETS]), na,
            kernel="qsim::elementwise_kernel<qsim::FloatShiftOp<false>, 3, 1>")
        g_host = W.lognormal_gradients().reshape(-1)
        for k in range(NSETS):
            a_in[k].copy_(torch.roll(torch.from_numpy(g_host).cuda(), 7654321 * k))
        run("float_e5m10_nearest_even_gradients", lambda k: Q.float_quantize(
            a_in[k % NSETS], 5, 10, Q.RN_EVEN, Q.SATURATE | Q.SUBNORMAL, out=a_out[k % NSETS]), na,
            kernel="qsim::elementwise_kernel<qsim::FloatGeneralOp, 0, 1>")
        # the same [128, 256, 56, 56] tensor with one shared exponent per channel (dimension 1)
        cn, cc, chw = 128, 256, 56 * 56
        # (block rows: the workspace is one the caller keeps for the shape, zero-filled once, so no call
        # launches anything but its one kernel; `gave_up_waiting` must stay 0 on an idle GPU)
        cws = torch.zeros(max(Q.block_workspace_bytes(na, cn, cc, chw), 16), dtype=torch.uint8, device="cuda")
        for mode, tag in ((Q.RN_EVEN, "nearest_even"), (Q.STOCHASTIC, "stochastic")):
            run(f"block8_per_channel_128x256x56x56_{tag}", lambda k, mode=mode: Q.block_quantize(
                a_in[k % NSETS], cn, cc, chw, 8, mode, Q.WORKSPACE_KEPT, 1234, k, out=a_out[k % NSETS], workspace=cws), na,
                extra={"note": "blocks along dimension 1; single pass, the workgroups of a channel meet among themselves"},
                kernel=f"qsim::block_cluster_strided_kernel<{mode}>")["gave_up_waiting"] = Q.workspace_timeouts(cws)
        del a_in, a_out, cws
        torch.cuda.empty_cache()
        # the same per channel where the feature map is not a whole number of groups: [128, 64, 55, 55]
        on, oc, ohw = 128, 64, 55 * 55
        o_in, o_out = _rotating(W.relu_activations((on, oc, 55, 55)).reshape(-1), torch)
        ows = torch.zeros(max(Q.block_workspace_bytes(on * oc * ohw, on, oc, ohw), 16), dtype=torch.uint8, device="cuda")
        for mode, tag in ((Q.RN_EVEN, "nearest_even"), (Q.STOCHASTIC, "stochastic")):
            run(f"block8_per_channel_128x64x55x55_{tag}", lambda k, mode=mode: Q.block_quantize(
                o_in[k % NSETS], on, oc, ohw, 8, mode, Q.WORKSPACE_KEPT, 1234, k, out=o_out[k % NSETS], workspace=ows), on * oc * ohw,
                extra={"note": "segments of 3025 elements: single pass over the tensor's own groups of four, shared edge groups masked"},
                kernel=f"qsim::block_cluster_ragged_kernel<{mode}>")["gave_up_waiting"] = Q.workspace_timeouts(ows)
        del o_in, o_out, ows
        torch.cuda.empty_cache()

        m_host = W.row_scaled_matrix()
        rows, cols = m_host.shape
        m_in = [torch.from_numpy(np.roll(m_host, 17 * k, axis=0)).cuda() for k in range(NSETS)]
        m_out = [torch.empty_like(m_in[0]) for _ in range(NSETS)]
        nm = rows * cols
        ws_bytes = Q.block_workspace_bytes(nm, 1, 1, nm)
        ws = torch.zeros(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
        for mode, tag in ((Q.RN_EVEN, "nearest_even"), (Q.STOCHASTIC, "stochastic")):
            run(f"block8_per_row_{tag}", lambda k, mode=mode: Q.block_quantize(
                m_in[k % NSETS], 1, rows, cols, 8, mode, 0, 1234, k, out=m_out[k % NSETS]), nm,
                kernel=f"qsim::block_cached_kernel<{mode}, 4, true, 256>")
            run(f"block8_whole_tensor_{tag}", lambda k, mode=mode: Q.block_quantize(
                m_in[k % NSETS], 1, 1, nm, 8, mode, Q.WORKSPACE_KEPT, 1234, k, out=m_out[k % NSETS], workspace=ws), nm,
                extra={"note": "single pass, one launch: 1024 resident workgroups hold the tensor in registers and meet once"},
                kernel=f"qsim::block_resident_kernel<{mode}, 16, false>")["gave_up_waiting"] = Q.workspace_timeouts(ws)
        # the same call from a caller that does not keep its workspace: a clearing launch goes first
        loose = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
        run("block8_whole_tensor_stochastic_workspace_not_kept", lambda k: Q.block_quantize(
            m_in[k % NSETS], 1, 1, nm, 8, Q.STOCHASTIC, 0, 1234, k, out=m_out[k % NSETS], workspace=loose), nm,
            extra={"note": "two launches: the workspace is cleared first"},
            kernel="qsim::block_sync_clear_kernel + qsim::block_resident_kernel<3, 16, false>")
        # one GPU's share of the same tensor split over two: block maxima of the share, the elementwise
        # maximum that stands in for the max-all-reduce, then quantize with the given maxima
        half = nm // 2
        other_max = Q.block_max(m_in[0].reshape(-1)[half:], 1, 1, nm - half, workspace=ws)
        share_max = torch.empty_like(other_max)

        def shard(k):
            x = m_in[k % NSETS].reshape(-1)[:half]
            Q.block_max(x, 1, 1, half, out=share_max, workspace=ws)
            torch.maximum(share_max, other_max, out=share_max)
            Q.block_quantize_with_max(x, 1, 1, half, 8, share_max, Q.STOCHASTIC, 0, 1234, k,
                                      out=m_out[k % NSETS].reshape(-1)[:half])

        run("block8_whole_tensor_one_of_two_shards_stochastic", shard, half,
            extra={"note": "block_max + maximum + block_quantize_with_max on half of the tensor: two passes, 12 B/element"},
            kernel="qsim::block_slice_max_kernel + qsim::block_fold_partials_wide_kernel + (torch maximum) + "
                   "qsim::block_slice_apply_kernel<3>")
        del m_in, m_out
        torch.cuda.empty_cache()

        w, g, m = W.sgd_state()
        npar = w.size
        fg = Q.Format(Q.KIND_FLOAT, 5, 2, Q.STOCHASTIC, Q.SATURATE | Q.SUBNORMAL)
        fm = Q.Format(Q.KIND_FIXED, 16, 12, Q.STOCHASTIC, Q.SATURATE)
        fw = Q.Format(Q.KIND_BLOCK, 8, 256, Q.RN_EVEN, 0)
        sets = []
        for k in range(NSETS):
            sets.append([torch.from_numpy(np.roll(a, 99991 * k)).cuda() for a in (w, g, m)] + [torch.empty(npar, device="cuda")])
        run("quant_sgd_step_25.6M", lambda k: Q.quant_sgd_step(sets[k % NSETS][0], sets[k % NSETS][1], sets[k % NSETS][2],
                                                               0.1, 0.9, fg, fm, fw, 1234, k + 2, w_q=sets[k % NSETS][3]),
            npar, bpe=SGD_BYTES_PER_PARAM,
            extra={"note": "grad float(5,2) stochastic, momentum fixed(16,12) stochastic, weight block8 per 256 nearest"},
            kernel="qsim::sgd_step_kernel<true>")
        del sets
        torch.cuda.empty_cache()

        # the same step over the 161 parameter tensors of a ResNet-50: one multi-tensor call against
        # one call per tensor
        sizes = W.resnet50_parameter_sizes()
        total = sum(sizes)
        flat = [torch.from_numpy(a[:total].copy()).cuda() for a in (w, g, m)] + [torch.empty(total, device="cuda")]
        lists = [list(torch.split(f, sizes)) for f in flat]
        table = Q.SgdTensorList(lists[0], lists[1], lists[2], lists[3])
        run("quant_sgd_step_table_resnet50_161_tensors", lambda k: table.step(0.1, 0.9, fg, fm, fw, 1234, k + 2), total,
            bpe=SGD_BYTES_PER_PARAM, extra={"note": "one call, one launch: the list is a table in device memory"},
            kernel="qsim::sgd_table_kernel<true>")
        run("quant_sgd_step_multi_resnet50_161_tensors", lambda k: table.step_batched(0.1, 0.9, fg, fm, fw, 1234, k + 2), total,
            bpe=SGD_BYTES_PER_PARAM, extra={"note": "one call, three launches of up to 64 tensors (pointer arrays)"},
            kernel="qsim::sgd_multi_kernel<true> x 3")

        def per_tensor(k):
            for t in range(len(sizes)):
                Q.quant_sgd_step(lists[0][t], lists[1][t], lists[2][t], 0.1, 0.9, fg, fm, fw, 1234, k + 2 + t, w_q=lists[3][t])

        run("quant_sgd_step_per_tensor_resnet50_161_calls", per_tensor, total, bpe=SGD_BYTES_PER_PARAM,
            kernel="qsim::sgd_step_kernel<true> x 161", launches=max(20, reps // 10))
        del flat, lists
        torch.cuda.empty_cache()
        result["formats"] = formats

    # ---- CPU baseline: the oracle as it stands, on the host cores ------------------------------
    if not args.no_cpu:
        from oracle import qsim_ref as R

        threads = min(16, os.cpu_count() or 1)
        R.lib()
        # whole passes over the headline tensor until about 15 s of CPU work have gone by
        passes, dt = 0, 0.0
        t0 = time.perf_counter()
        while passes < 50 and dt * threads < 15.0:
            R.fixed_quantize(x_host, 8, 6, R.STOCHASTIC, R.SATURATE, seed=1234, stream_id=passes, threads=threads)
            passes += 1
            dt = time.perf_counter() - t0
        # and one thread alone, on the first eighth of the tensor
        part = x_host[: n // 8]
        t0 = time.perf_counter()
        R.fixed_quantize(part, 8, 6, R.STOCHASTIC, R.SATURATE, seed=1234, stream_id=0, threads=1)
        one = part.size / (time.perf_counter() - t0)
        result["cpu_baseline"] = {"value": n * passes / dt, "unit": "elements/s", "cores": threads, "kind": "oracle",
                                  "threads": threads, "host_cores": os.cpu_count(),
                                  "note": "a GPU box gives one GPU's job 16 cores, whatever the host has: the oracle runs on "
                                          "min(16, host cores) threads, and `cores` is that number",
                                  "sample": f"{passes} passes over the whole {n}-element tensor of the headline workload, "
                                            f"each split over {threads} threads ({dt:.2f} s wall, "
                                            f"{dt * threads:.0f} s of CPU work)",
                                  "single_thread_value": one}
        if not args.no_formats:
            # the oracle on samples of the other workloads (elements/s; block and SGD entries run on one thread)
            def rate(fn, count):
                t0 = time.perf_counter()
                fn()
                return count / (time.perf_counter() - t0)

            acts = W.relu_activations((8, 256, 56, 56)).reshape(-1)
            grads = W.lognormal_gradients((8, 256, 56, 56)).reshape(-1)
            mat = W.row_scaled_matrix(512, 4096)
            w, g, m = W.sgd_state(1 << 21)
            fg, fm, fw = R.Format(1, 5, 2, 3, 3), R.Format(2, 16, 12, 3, 1), R.Format(3, 8, 256, 0, 0)
            result["cpu_baseline"]["other_formats"] = {
                "float_e8m7_stochastic_activations": rate(lambda: R.float_quantize(
                    acts, 8, 7, R.STOCHASTIC, R.SATURATE | R.SUBNORMAL, seed=1234, threads=threads), acts.size),
                "float_e5m10_nearest_even_gradients": rate(lambda: R.float_quantize(
                    grads, 5, 10, R.RN_EVEN, R.SATURATE | R.SUBNORMAL, threads=threads), grads.size),
                "block8_per_row_stochastic_one_thread": rate(lambda: R.block_quantize(
                    mat, 1, mat.shape[0], mat.shape[1], 8, R.STOCHASTIC, 0, 1234, 0), mat.size),
                "block8_whole_tensor_nearest_even_one_thread": rate(lambda: R.block_quantize(
                    mat, 1, 1, mat.size, 8, R.RN_EVEN), mat.size),
                "quant_sgd_step_one_thread": rate(lambda: R.quant_sgd_step(w, g, m, 0.1, 0.9, fg, fm, fw, 1234, 2), w.size),
            }
    print(json.dumps(result), flush=True)
    # leave nothing behind: everything queued has finished, and the tensors that are still alive go
    # back now rather than in the interpreter's teardown
    torch.cuda.synchronize()
    x_host = None
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    sys.exit(main())
