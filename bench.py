#!/usr/bin/env python3
"""HGEMM benchmark on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload ALL|C1|C2|C3|C4|C5|P] [--cold] ...

Default (no flags, workload ALL) -- the metric itself.  A step is one pass of the whole hot path
(plans made beforehand, then one hgemm_run per shape) over every shape of
  C4  the 200-shape grid over {64..12288}^3, uniform[-1,1]            -> `value` = geomean TFLOP/s
  C2  the square sweep 1024^3 .. 8192^3, N(0,1)/sqrt(K)               (warm, as C4)
  C5  16384 x 16384 x {8192, 16384}, uniform[-1,1]                    (warm)
  C3  the 20 LLM-projection skinny shapes, A~N(0,1), B~N(0,0.02^2)    (cold: operand sets rotate
      through > 768 MiB, so every call streams its weights from HBM)
with all operands resident in HBM before the timed region.  After W untimed steps exactly K steps are
timed between device synchronisations.  The K steps run shape-major: a shape's K calls go back to back
on the stream (the paper's offline mode, Section 2.4.2) in five batches, each between its own pair of
events on that stream (Section 2.4.1), so mean, median and minimum per-call times are real statistics
of five measurements (with K < 50: one batch, one event pair around the K calls, mean only).  With --graph each batch is captured once in a HIP graph and replayed instead
(no host enqueue cost; pays only with long batches).  The last line printed is one JSON object:

  value         geometric mean over the 200 grid shapes of 2*M*N*K / (mean time per call), TFLOP/s
  workloads     geomean and aggregate TFLOP/s of each of the four workloads
  roofline      the dominant kernel (the launch with the largest share of a step; matrix-core bound)
                against the published fp16 MFMA peak
  roofline_hbm  the memory-bound skinny shapes (M <= 128 of C3, cold) against the published HBM peak:
                best, median and count at or above 60 %
  cpu_baseline  the CPU oracle timed on a bounded sample of the workload on this host

With --workload C1..C5 a single workload is timed (numpy-drawn inputs, as in the parity tests);
"--cold" rotates operand sets so that the 256 MiB last-level cache cannot hold them (the server-mode
effect of Section 2.4.2); "--server" is server mode itself; P is the paper's 1000-shape grid.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP16_TFLOPS = 2500.0      # MI355X dense fp16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published

# Bytes per launch between the L2s and the memory side (last-level cache + HBM), NOT measured by this
# program: copied from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this program, scaled by kernels of
# known size (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0); figures and commands in profiles/.  Reported as
# roofline.traffic with roofline.traffic_source saying so.
PROFILED_TRAFFIC_BYTES = {
    (1024, 1024, 1024): (6188.0 * 2.0 + 2048.0) * 1024,
    (2048, 2048, 2048): (24633.0 * 2.0 + 8192.0) * 1024,
    (4096, 4096, 4096): (147517.0 * 2.0 + 32768.0) * 1024,
    (8192, 8192, 8192): (786489.6 * 2.0 + 131072.0) * 1024,
    (16384, 16384, 8192): (3152703.9 * 2.0 + 532480.1) * 1024,
    (16384, 16384, 16384): (6937502.9 * 2.0 + 532480.0) * 1024,
    # cold skinny shapes (the HBM roofline's candidates); sums over the kernels of one call
    (1, 4096, 4096): (16498.6 * 2.0 + 146.0) * 1024,
    (16, 4096, 4096): (17723.5 * 2.0 + 1664.0) * 1024,
    (1, 11008, 4096): (44214.7 * 2.0 + 372.2) * 1024,
    (16, 11008, 4096): (45994.0 * 2.0 + 3096.0) * 1024,
    (1, 4096, 11008): (44201.6 * 2.0 + 146.0) * 1024,
    (16, 4096, 11008): (45982.9 * 2.0 + 1152.0) * 1024,
    (1, 14336, 4096): (57415.4 * 2.0 + 28.0) * 1024,
    (16, 14336, 4096): (57895.3 * 2.0 + 448.0) * 1024,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="ALL", choices=["ALL", "C1", "C2", "C3", "C3L", "C3O", "C4", "C5", "P"],
                    help="ALL: the metric (grid C4 as the value, C2, C5 warm and C3 cold beside it); C1..C5: one "
                         "benchmark configuration; C3L, C3O: the C3 kind of shape for a model four times the size and for other "
                         "model widths (use with --cold); P: the paper's full grid, all 1000 triples over "
                         "{64..16384}^3 (Abstract), timed shape by shape beside torch.matmul")
    ap.add_argument("--cold", action="store_true", help="rotate operand sets so caches are cold")
    ap.add_argument("--shapes", default="", help="with --workload C2..C5: time these shapes (MxNxK,MxNxK,...) instead of the workload's own, "
                                                 "inputs drawn by the workload's recipe, kernels chosen by hgemm_plan (shapes outside the "
                                                 "dispatch table: nearest tuned shape or cost model)")
    ap.add_argument("--layout", default="nn", choices=["nn", "tn"],
                    help="nn: B row-major (K x N); tn: B column-major, stored N x K (Section 2.2.2)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--spec", default=None, help="force one specialisation for every shape (tuning aid)")
    ap.add_argument("--table", action="store_true", help="print the per-shape table to stderr")
    ap.add_argument("--server", action="store_true",
                    help="server mode (Section 2.4.2): calls separated by random idle gaps of 0-2 ms, each call "
                         "bracketed by its own events; the gaps are not part of any reported time")
    ap.add_argument("--per-call-events", action="store_true",
                    help="bracket every call with its own event pair (adds the event/launch gap to every call)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run the roofline calibration kernels (MFMA-only loop, 1 GiB streaming read, "
                         "128 MiB fill) -- kernels of known size for scaling profiler counters")
    ap.add_argument("--order", choices=["flop", "listed"], default="flop",
                    help="default run: order of the shapes inside a step -- by ascending 2*M*N*K, so that a shape runs after "
                         "shapes of similar power draw (the chip carries a large problem's throttled clock into the next "
                         "milliseconds), or as the workloads list them")
    ap.add_argument("--graph", action="store_true",
                    help="capture each shape's K back-to-back calls in a HIP graph and time its replay: removes the "
                         "host's enqueue rate (about 3.4 us per call from Python) from launch-bound small shapes")
    ap.add_argument("--library-context", action="store_true",
                    help="also time torch.matmul (the vendor GEMM library the PyTorch build ships) on the same "
                         "operands with the same protocol; context only, the library under test never calls it")
    return ap.parse_args()


def workload_shapes(name):
    import workloads as wl

    if name == "C1":
        return [wl.C1_SHAPE], lambda s: wl.c1_inputs()
    if name == "C2":
        return list(wl.C2_SHAPES), wl.c2_inputs
    if name == "C3":
        return list(wl.C3_SHAPES), wl.c3_inputs
    if name == "C3L":
        return list(wl.C3_LARGE_SHAPES), wl.c3_inputs
    if name == "C3O":
        return list(wl.C3_OTHER_SHAPES), wl.c3_inputs
    if name == "C4":
        return wl.c4_shapes(), wl.c4_inputs
    return list(wl.C5_SHAPES), wl.c5_inputs


def cpu_baseline():
    """The oracle as it stands, on a bounded sample of the default workload."""
    import numpy as np

    import workloads as wl
    from oracle import hgemm_oracle as orc

    rows = 2048
    a1, b1 = wl.c2_inputs((1024, 1024, 1024))
    a2, b2 = wl.c2_inputs((2048, 2048, 2048))
    a3, b3 = wl.c2_inputs((4096, 4096, 4096))
    a3 = np.ascontiguousarray(a3[:rows])
    t0 = time.perf_counter()
    orc.hgemm(a1, b1)
    orc.hgemm(a2, b2)
    orc.hgemm(a3, b3)
    dt = time.perf_counter() - t0
    flop = 2.0 * 1024 ** 3 + 2.0 * 2048 ** 3 + 2.0 * rows * 4096 * 4096
    return {
        "value": flop / dt * 1e-12,
        "unit": "TFLOP/s",
        "cores": orc.threads(),
        "kind": "oracle",
        "sample": "oracle on the full 1024^3 and 2048^3 products plus the first 2048 rows of the 4096^3 product "
                  f"of the square sweep ({dt:.1f} s of CPU work)",
    }


def paper_grid(args):
    """The paper's own workload (Abstract, Section 3): every (M, N, K) in {64, ..., 16384}^3, offline mode, and
    its headline figure -- the mean over shapes of the speedup against the vendor library -- measured here against
    torch.matmul on the same operands.  Operands are drawn on the device (uniform[-1,1], seed per shape): a
    thousand operand sets do not fit HBM at once, so each shape is allocated, timed and freed in turn."""
    import numpy as np
    import torch

    import paper_2512_02551_amd as hg
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    hg.load()
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    v = wl.PAPER_GRID_VALUES
    shapes = [(m, n, k) for m in v for n in v for k in v]
    rows = []
    t_wall = time.perf_counter()
    for (M, N, K) in shapes:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(M * 1000003 + N * 1009 + K)
        a = (torch.rand((M, K), device="cuda", generator=gen) * 2 - 1).half()
        b = (torch.rand((K, N), device="cuda", generator=gen) * 2 - 1).half()
        c = torch.empty((M, N), device="cuda", dtype=torch.float16)
        c_lib = torch.empty_like(c)
        tn = args.layout == "tn"
        if tn:                                    # the same matrix stored N x K (column-major B, Section 2.2.2)
            b = b.t().contiguous()
        b_lib = b.t() if tn else b                # torch.matmul sees the strides and dispatches the library's TN kernel
        flop = 2.0 * M * N * K
        steps = max(2, min(args.steps, int(2e12 / flop) + 2))          # a few milliseconds of work per measurement
        warm = max(1, min(args.warmup, steps))
        plan = hg.Plan(M, N, K, hg.Layouts.make(b_col_major=True) if tn else None)

        def ours(n):
            for _ in range(n):
                plan.run(a.data_ptr(), b.data_ptr(), c.data_ptr(), sh)

        def lib(n):
            for _ in range(n):
                torch.matmul(a, b_lib, out=c_lib)

        t = {}
        for name, fn in (("ours", ours), ("lib", lib)):
            fn(warm)
            torch.cuda.synchronize()
            replay = None
            if args.graph:                       # both sides as graph replays: no host enqueue cost on either
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    if name == "ours":
                        cs = torch.cuda.current_stream().cuda_stream
                        for _ in range(steps):
                            plan.run(a.data_ptr(), b.data_ptr(), c.data_ptr(), cs)
                    else:
                        fn(steps)
                replay = g.replay
                replay()
                torch.cuda.synchronize()
            best = float("inf")
            for _ in range(3):                                              # best of three batches
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                if replay:
                    replay()
                else:
                    fn(steps)
                e1.record(stream)
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1) / steps)
            t[name] = best
        rows.append({"shape": [M, N, K], "spec": plan.describe(), "us": t["ours"] * 1e3, "tflops": flop / t["ours"] * 1e-9,
                     "lib_us": t["lib"] * 1e3, "speedup_vs_lib": t["lib"] / t["ours"]})
        plan.destroy()
        del a, b, c, c_lib
        if args.table:
            r = rows[-1]
            print("{:>18s} {:10.1f} us {:8.1f} TFLOP/s  torch.matmul {:10.1f} us  x{:.2f}  {}".format(
                "x".join(map(str, r["shape"])), r["us"], r["tflops"], r["lib_us"], r["speedup_vs_lib"], r["spec"]), file=sys.stderr)
    wall = time.perf_counter() - t_wall
    sp = np.array([r["speedup_vs_lib"] for r in rows])
    tf = np.array([r["tflops"] for r in rows])
    out = {
        "metric": "HGEMM TFLOP/s geomean over (M,N,K) grid", "value": float(np.exp(np.log(tf).mean())), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16 inputs/outputs, f32 accumulate", "data": "synthetic",
        "config": {"workload": "the paper's grid: 1000 triples over {64,...,16384}^3, uniform[-1,1], offline mode",
                   "layout": "TN (B column-major)" if args.layout == "tn" else "NN row-major", "cache": "warm",
                   "timing": ("best of three replays of a graph of back-to-back calls per shape (library too)" if args.graph else
                              "best of three batches of back-to-back calls per shape")},
        "library_context": {
            "what": "torch.matmul of this PyTorch build on the same operands and protocol (context only)",
            "mean_speedup": float(sp.mean()), "geomean_speedup": float(np.exp(np.log(sp).mean())),
            "win_rate": float((sp > 1.0).mean()), "min_speedup": float(sp.min()), "max_speedup": float(sp.max()),
            "mean_speedup_of_max_with_library": float(np.maximum(sp, 1.0).mean()),
        },
        "arithmetic_mean_tflops": float(tf.mean()),
        "per_shape": rows,
    }
    print(json.dumps(out))


def metric_run(args):
    """The default run: the 200-shape grid (the metric's value) with the square sweep, the two large
    shapes and the cold skinny shapes beside it, one timed region."""
    import numpy as np
    import torch

    import paper_2512_02551_amd as hg
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    hg.load()          # fails loudly if libhgemm.so is missing: there is no fallback path
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    steps, warmup = max(1, args.steps), max(0, args.warmup)
    # An event record between batches costs the stream about 4 us (measured: 3.4 us per call of a 2.4 us
    # kernel in batches of 4, 2.8 in batches of 10), so a batch holds at least 10 calls.  With at least 50
    # steps a shape's calls go in five batches and the median and minimum over them are reported; with
    # fewer they go in one batch (one event pair around all K calls) and those two fields are null.
    n_batches = 5 if steps >= 50 else 1
    batch_sizes = [steps // n_batches + (1 if i < steps % n_batches else 0) for i in range(n_batches)]

    jobs = [("C4", s, False) for s in wl.c4_shapes()] + [("C2", s, False) for s in wl.C2_SHAPES] + \
           [("C5", s, False) for s in wl.C5_SHAPES] + [("C3", s, True) for s in wl.C3_SHAPES]
    if args.order == "flop":
        jobs.sort(key=lambda j: 2.0 * j[1][0] * j[1][1] * j[1][2])     # stable: equal sizes keep their listed order
    sets = []
    for (cfg, (M, N, K), cold) in jobs:
        a, b = wl.device_inputs(cfg, (M, N, K))
        n_sets = 1
        if cold:
            per_set = 2 * (M * K + K * N + M * N)
            n_sets = max(2, min(64, math.ceil(768 * 2 ** 20 / per_set)))
        bufs = [(a if i == 0 else a.clone(), b if i == 0 else b.clone(), torch.empty((M, N), dtype=torch.float16, device="cuda"))
                for i in range(n_sets)]
        plan = hg.Plan(M, N, K, None, None)
        sets.append({"cfg": cfg, "shape": (M, N, K), "cold": cold, "bufs": bufs, "plan": plan, "desc": plan.describe(),
                     "info": plan.launch_info(), "next": 0})
    torch.cuda.synchronize()

    # A batch of back-to-back calls is enqueued by one hgemm_run_many (device pointers marshalled once):
    # the 2-3 us kernels of the small grid shapes are otherwise timed at the speed of the interpreter.
    for s in sets:
        s["ptrs"] = s["plan"].pointer_sets([(a.data_ptr(), b.data_ptr(), c.data_ptr()) for (a, b, c) in s["bufs"]])

    def calls(s, count, sh=sh):
        # one hgemm_run_many per batch: the loop over the calls is the library's, not the interpreter's
        s["plan"].run_many(count, s["ptrs"], sh, s["next"] % s["ptrs"][0])
        s["next"] += count

    for s in sets:
        calls(s, warmup)
    torch.cuda.synchronize()

    def timed_region(launch_batch):
        """All shapes, shape-major, five batches each; consecutive batches share the event between them (six
        records per shape, not ten: a record costs about as much as one of the small kernels).  Returns
        (per shape, per batch (start, end) events, wall seconds)."""
        marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(batch_sizes) + 1)] for _ in sets]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for si, s in enumerate(sets):
            marks[si][0].record(stream)
            for bi, count in enumerate(batch_sizes):
                launch_batch(si, s, bi, count)
                marks[si][bi + 1].record(stream)
        torch.cuda.synchronize()
        wall_s = time.perf_counter() - t0
        return [[(m[bi], m[bi + 1]) for bi in range(len(batch_sizes))] for m in marks], wall_s

    if not args.graph:
        # the paper's offline mode as it stands: every call enqueued from the host, back to back
        events, wall = timed_region(lambda si, s, bi, count: calls(s, count))
    else:
        # each batch captured once in a HIP graph (hgemm_run only launches kernels on the stream it is
        # given) and replayed between the batch's events: no host enqueue cost at all, but a graph launch
        # costs several microseconds itself, so this pays only with long batches (--steps of 200 and more)
        graphs = []
        for s in sets:
            per_batch = []
            for count in batch_sizes:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    calls(s, count, torch.cuda.current_stream().cuda_stream)
                per_batch.append(g)
            graphs.append(per_batch)
        torch.cuda.synchronize()
        events, wall = timed_region(lambda si, s, bi, count: graphs[si][bi].replay())

    ridge = PEAK_FP16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    per_shape = []
    for si, s in enumerate(sets):
        M, N, K = s["shape"]
        flop = 2.0 * M * N * K
        byts = 2.0 * (M * K + K * N + M * N)
        total_ms = sum(e0.elapsed_time(e1) for (e0, e1) in events[si])
        per_call = np.array([e0.elapsed_time(e1) / c for (e0, e1), c in zip(events[si], batch_sizes)])
        mean_ms = total_ms / steps
        per_shape.append({
            "workload": s["cfg"] + (" cold" if s["cold"] else ""), "shape": [M, N, K], "spec": s["desc"],
            "workgroups": s["info"]["workgroups"],
            "mean_us": mean_ms * 1e3,
            "median_us": float(np.median(per_call)) * 1e3 if n_batches >= 5 else None,
            "min_us": float(per_call.min()) * 1e3 if n_batches >= 5 else None,
            "tflops": flop / mean_ms * 1e-9, "gbs": byts / mean_ms * 1e-6,
            "frac_mfma_peak": flop / mean_ms * 1e-9 / PEAK_FP16_TFLOPS,
            "frac_hbm_peak": byts / mean_ms * 1e-6 / PEAK_HBM_GBS,
            "ai_flop_per_byte": flop / byts,
        })

    def summary(rows):
        fl = sum(2.0 * r["shape"][0] * r["shape"][1] * r["shape"][2] for r in rows)
        us = sum(r["mean_us"] for r in rows)
        return {"shapes": len(rows), "geomean_tflops": math.exp(sum(math.log(r["tflops"]) for r in rows) / len(rows)),
                "aggregate_tflops": fl / us * 1e-6, "us_per_step": us}

    groups = {}
    for r in per_shape:
        groups.setdefault(r["workload"], []).append(r)
    workloads = {name: summary(rows) for name, rows in groups.items()}

    # matrix-core roofline: the launch with the largest share of a step
    dom = max(per_shape, key=lambda p: p["mean_us"])
    M, N, K = dom["shape"]
    roofline = {"bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s",
                "frac": dom["tflops"] / PEAK_FP16_TFLOPS, "traffic": PROFILED_TRAFFIC_BYTES.get((M, N, K)),
                "kernel": f"{M}x{N}x{K} [{dom['spec']}]", "avg_launch_us": dom["mean_us"],
                "flop_per_launch": 2.0 * M * N * K}
    roofline["traffic_source"] = ("rocprofv3 FETCH_SIZE/WRITE_SIZE of an earlier run of this command, see profiles/"
                                  if roofline["traffic"] else None)
    assert dom["ai_flop_per_byte"] >= ridge
    # HBM roofline: the memory-bound skinny shapes (arithmetic intensity below the ridge), streamed from HBM
    mem = sorted((r for r in groups["C3 cold"] if r["ai_flop_per_byte"] < ridge and r["shape"][0] <= 128),
                 key=lambda r: r["frac_hbm_peak"])
    best, med = mem[-1], mem[len(mem) // 2]

    def hbm_obj(r):
        m, n, k = r["shape"]
        return {"bound": "hbm", "achieved": r["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": r["frac_hbm_peak"],
                "traffic": PROFILED_TRAFFIC_BYTES.get((m, n, k)), "kernel": f"{m}x{n}x{k} [{r['spec']}]",
                "avg_launch_us": r["mean_us"], "bytes_per_launch": 2.0 * (m * k + k * n + m * n)}

    roofline_hbm = hbm_obj(best)
    roofline_hbm["median"] = hbm_obj(med)
    roofline_hbm["memory_bound_shapes"] = len(mem)
    roofline_hbm["at_or_above_60pct"] = sum(1 for r in mem if r["frac_hbm_peak"] >= 0.60)
    roofline_hbm["per_shape_frac"] = {"x".join(map(str, r["shape"])): round(r["frac_hbm_peak"], 4) for r in mem}

    if args.table:
        for p in per_shape:
            print("{:8s} {:>18s}  {:9.1f} us (median {:9.1f}, min {:9.1f})  {:8.1f} TFLOP/s ({:4.1f}% MFMA)  {:8.1f} GB/s ({:4.1f}% HBM)  {}".format(
                p["workload"], "x".join(map(str, p["shape"])), p["mean_us"], p["median_us"] or float("nan"), p["min_us"] or float("nan"), p["tflops"],
                100 * p["frac_mfma_peak"], p["gbs"], 100 * p["frac_hbm_peak"], p["spec"]), file=sys.stderr)

    out = {
        "metric": "HGEMM TFLOP/s geomean over (M,N,K) grid; % of FP16 MFMA peak / HBM BW",
        "value": workloads["C4"]["geomean_tflops"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": wall / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 inputs/outputs, f32 accumulate",
        "data": "synthetic",
        "config": {
            "workload": "C4: 200-shape grid sampled with seed 1 from {64..12288}^3, uniform[-1,1] (the value); timed in the "
                        "same steps: C2 square sweep and C5 16384^2 x {8192,16384} warm, C3 LLM skinny shapes from HBM (cold)",
            "layout": "NN row-major", "cache": "warm (C3: cold, rotating operand sets > 768 MiB)",
            "order": "shapes by ascending 2*M*N*K" if args.order == "flop" else "shapes as the workloads list them",
            "timing": (f"{steps} back-to-back calls per shape in {n_batches} batches, an event on the launch stream between batches; " +
                       ("each batch captured once in a HIP graph and replayed" if args.graph else "calls enqueued one by one from the host")),
            "aggregate_tflops": sum(2.0 * r["shape"][0] * r["shape"][1] * r["shape"][2] for r in per_shape) * steps / wall * 1e-12,
        },
        "workloads": workloads,
        "roofline": roofline,
        "roofline_hbm": roofline_hbm,
        "per_shape": per_shape,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    for s in sets:
        s["plan"].destroy()
    print(json.dumps(out))


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build measures one GPU only (asked for --gpus {args.gpus}); "
              "the library has no multi-GPU path (each GPU would run it on its own block of C)", file=sys.stderr)
        sys.exit(2)

    if args.shapes and args.workload in ("ALL", "P", "C1"):
        sys.exit("bench.py: --shapes needs --workload C2, C3, C3L, C3O, C4 or C5 (whose input recipe it uses)")
    if args.workload == "P":
        paper_grid(args)
        return
    if args.workload == "ALL":
        if args.cold or args.server or args.per_call_events or args.spec or args.layout != "nn" or args.library_context or args.calibrate:
            print("bench.py: these options need a single workload (--workload C1..C5)", file=sys.stderr)
            sys.exit(2)
        metric_run(args)
        return

    import numpy as np
    import torch

    import paper_2512_02551_amd as hg

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    hg.load()          # fails loudly if libhgemm.so is missing: there is no fallback path

    shapes, make_inputs = workload_shapes(args.workload)
    if args.shapes:
        if args.workload not in ("C2", "C3", "C3L", "C3O", "C4", "C5"):
            sys.exit("bench.py: --shapes needs --workload C2, C3, C4 or C5 (whose input recipe it uses)")
        shapes = [tuple(int(v) for v in item.split("x")) for item in args.shapes.split(",") if item]
        if any(len(sh_) != 3 or min(sh_) < 1 for sh_ in shapes):
            sys.exit("bench.py: --shapes takes MxNxK,MxNxK,... with positive sizes")

    # operands resident in HBM before anything is timed
    def upload(x):
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.float16)

    sets = []
    for (M, N, K) in shapes:
        a, b = make_inputs((M, N, K))
        n_sets = 1
        if args.cold:
            per_set = 2 * (M * K + K * N + M * N)
            n_sets = max(2, min(64, math.ceil(768 * 2 ** 20 / per_set)))
        group = []
        if args.layout == "tn":
            b = np.ascontiguousarray(b.T)
        da, db = upload(a), upload(b)
        for i in range(n_sets):
            group.append((da if i == 0 else da.clone(), db if i == 0 else db.clone(),
                          torch.empty((M, N), dtype=torch.float16, device="cuda")))
        plan = hg.Plan(M, N, K, hg.Layouts.make(b_col_major=(args.layout == "tn")), args.spec)
        sets.append({"shape": (M, N, K), "bufs": group, "plan": plan, "desc": plan.describe(),
                     "info": plan.launch_info()})
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    # Timed region.  The K steps are run shape-major: every shape's K calls go back to back on the
    # stream between one pair of events (the paper's offline mode, Section 2.4.2: kernels executed
    # consecutively without pauses), so a per-call time is that pair's elapsed time / K and carries no
    # event or launch gap.  With --cold the K calls rotate through operand sets whose total exceeds the
    # last-level cache.  "--per-call-events" brackets every single call instead.
    import random
    gap_rng = random.Random(0)
    if args.server:
        args.per_call_events = True

    # entry point bound once, device pointers taken once: the enqueue loop of the small shapes is
    # otherwise timed at the speed of the interpreter
    hgemm_run = hg.load().hgemm_run
    for s in sets:
        s["ptrs"] = [(a.data_ptr(), b.data_ptr(), c.data_ptr()) for (a, b, c) in s["bufs"]]
        s["many"] = s["plan"].pointer_sets(s["ptrs"])
        s["handle"] = s["plan"]._h

    def run_shape(s, k0, count, events=None, sh=sh):
        ptrs, h = s["ptrs"], s["handle"]
        n = len(ptrs)
        if events is None:
            # one hgemm_run_many per batch: the loop over the calls is the library's, not the interpreter's
            s["plan"].run_many(count, s["many"], sh, k0 % n)
            return
        for k in range(count):
            a, b, c = ptrs[(k0 + k) % n]
            if args.server:
                torch.cuda.synchronize()                       # the device is idle during the gap
                time.sleep(gap_rng.uniform(0.0, 2e-3))
            events[k][0].record(stream)
            if hgemm_run(h, a, b, c, sh):
                raise RuntimeError("hgemm_run failed")
            events[k][1].record(stream)

    for s in sets:
        run_shape(s, 0, args.warmup)
    torch.cuda.synchronize()

    # five batches per shape, each between its own event pair: mean, median and minimum are real statistics
    n_batches = 1 if args.graph else (min(5, args.steps) if args.per_call_events else (5 if args.steps >= 50 else 1))
    batch_sizes = [args.steps // n_batches + (1 if i < args.steps % n_batches else 0) for i in range(n_batches)]
    pair = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in batch_sizes] for _ in sets]
    per_call = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
                for _ in sets] if args.per_call_events else None
    graphs = None
    if args.graph:
        if per_call:
            print("bench.py: --graph times whole replays; it cannot be combined with per-call events", file=sys.stderr)
            sys.exit(2)
        graphs = []
        for s in sets:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                run_shape(s, args.warmup, args.steps, None, torch.cuda.current_stream().cuda_stream)
            g.replay()                              # one untimed replay
            graphs.append(g)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for si, s in enumerate(sets):
        done = 0
        for bi, count in enumerate(batch_sizes):
            pair[si][bi][0].record(stream)
            if graphs:
                graphs[si].replay()
            else:
                run_shape(s, args.warmup + done, count, per_call[si][done:done + count] if per_call else None)
            pair[si][bi][1].record(stream)
            done += count
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    per_shape = []
    for si, s in enumerate(sets):
        M, N, K = s["shape"]
        flop = 2.0 * M * N * K
        byts = 2.0 * (M * K + K * N + M * N)
        if per_call:
            ts = np.array([e0.elapsed_time(e1) for (e0, e1) in per_call[si]])
            mean_ms, med_ms, min_ms = float(ts.mean()), float(np.median(ts)), float(ts.min())
        else:
            ts = np.array([e0.elapsed_time(e1) / c for (e0, e1), c in zip(pair[si], batch_sizes)])
            mean_ms = float(sum(e0.elapsed_time(e1) for (e0, e1) in pair[si])) / args.steps
            # median and minimum are statistics over batches of at least ten calls; not reported below five batches
            med_ms, min_ms = (float(np.median(ts)), float(ts.min())) if len(ts) >= 5 else (None, None)
        per_shape.append({
            "shape": [M, N, K], "spec": s["desc"], "workgroups": s["info"]["workgroups"],
            "mean_us": mean_ms * 1e3, "median_us": med_ms and med_ms * 1e3, "min_us": min_ms and min_ms * 1e3,
            "tflops": flop / mean_ms * 1e-9, "gbs": byts / mean_ms * 1e-6,
            "frac_mfma_peak": flop / mean_ms * 1e-9 / PEAK_FP16_TFLOPS,
            "frac_hbm_peak": byts / mean_ms * 1e-6 / PEAK_HBM_GBS,
            "ai_flop_per_byte": flop / byts,
        })
    geomean = math.exp(sum(math.log(p["tflops"]) for p in per_shape) / len(per_shape))
    total_flop = sum(2.0 * m * n * k for (m, n, k) in shapes)

    # dominant kernel: the launch with the largest share of the step
    dom = max(per_shape, key=lambda p: p["mean_us"])
    M, N, K = dom["shape"]
    ridge = PEAK_FP16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    if dom["ai_flop_per_byte"] >= ridge:
        roofline = {"bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_FP16_TFLOPS, "unit": "TFLOP/s",
                    "frac": dom["tflops"] / PEAK_FP16_TFLOPS}
    else:
        roofline = {"bound": "hbm", "achieved": dom["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": dom["gbs"] / PEAK_HBM_GBS}
    roofline["traffic"] = PROFILED_TRAFFIC_BYTES.get((M, N, K))
    roofline["traffic_source"] = "rocprofv3 counters of an earlier run of this command, see profiles/" if roofline["traffic"] else None
    roofline["kernel"] = f"{M}x{N}x{K} [{dom['spec']}]"
    roofline["avg_launch_us"] = dom["mean_us"]

    if args.table:
        for p in per_shape:
            print("{:>18s}  {:9.1f} us  {:8.1f} TFLOP/s ({:4.1f}% MFMA)  {:8.1f} GB/s ({:4.1f}% HBM)  {}".format(
                "x".join(map(str, p["shape"])), p["mean_us"], p["tflops"], 100 * p["frac_mfma_peak"], p["gbs"],
                100 * p["frac_hbm_peak"], p["spec"]), file=sys.stderr)

    out = {
        "metric": "HGEMM TFLOP/s geomean over (M,N,K) grid",
        "value": geomean,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 inputs/outputs, f32 accumulate",
        "data": "synthetic",
        "config": {
            "workload": {"C1": "single 256^3, uniform[-1,1]",
                         "C2": "square HGEMM sweep M=N=K in {1024,2048,4096,8192}, entries N(0,1)/sqrt(K)",
                         "C3": "LLM-projection skinny shapes, A~N(0,1), B~N(0,0.02^2)",
                         "C3O": "LLM-projection skinny shapes of other model widths (M in {1,16,64,128,512}; 5120/13824/15360, 6144x4096, "
                                "10240x8192; beyond the five configurations), A~N(0,1), B~N(0,0.02^2)",
                         "C3L": "LLM-projection skinny shapes of a larger model (M in {1,16,64}, widths 8192 and 28672; beyond the five "
                                "configurations), A~N(0,1), B~N(0,0.02^2)",
                         "C4": "200-shape grid from {64..12288}^3, uniform[-1,1]",
                         "C5": "16384x16384x{8192,16384}, uniform[-1,1]"}[args.workload] + (
                             " -- shapes from the command line, this recipe's inputs" if args.shapes else ""),
            "layout": "NN row-major" if args.layout == "nn" else "TN (B column-major)", "cache": "cold" if args.cold else "warm",
            "timing": ("server mode: random idle gaps, per-call events" if args.server else
                       "per-call events" if args.per_call_events else
                       "replay of a HIP graph holding K back-to-back calls per shape" if args.graph else
                       f"K back-to-back calls per shape in {n_batches} batches, one event pair per batch"),
            "aggregate_tflops": total_flop * args.steps / wall * 1e-12,
        },
        "roofline": roofline,
        "per_shape": per_shape,
    }
    if args.library_context:
        # Context, as the paper quotes its kernels beside the vendor library (Section 2.2): same operands,
        # same back-to-back protocol, output into a preallocated tensor.
        lib_rows = []
        for s in sets:
            M, N, K = s["shape"]
            outs = [torch.empty_like(c) for (_, _, c) in s["bufs"]]

            def lib_calls(k0, count):
                for k in range(count):
                    a, b, _ = s["bufs"][(k0 + k) % len(s["bufs"])]
                    torch.matmul(a, b.t() if args.layout == "tn" else b, out=outs[(k0 + k) % len(outs)])

            lib_calls(0, args.warmup)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            lib_calls(args.warmup, args.steps)
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / args.steps
            lib_rows.append({"shape": [M, N, K], "mean_us": ms * 1e3, "tflops": 2.0 * M * N * K / ms * 1e-9,
                             "gbs": 2.0 * (M * K + K * N + M * N) / ms * 1e-6})
            del outs
        out["library_context"] = {
            "what": "torch.matmul of this PyTorch build on the same operands and protocol (context only)",
            "geomean_tflops": math.exp(sum(math.log(r["tflops"]) for r in lib_rows) / len(lib_rows)),
            "per_shape": lib_rows,
        }
        if args.table:
            for r, p in zip(lib_rows, per_shape):
                print("{:>18s}  torch.matmul {:9.1f} us {:8.1f} TFLOP/s {:8.1f} GB/s   torch.matmul time / this library's time = {:.2f}".format(
                    "x".join(map(str, r["shape"])), r["mean_us"], r["tflops"], r["gbs"], r["mean_us"] / p["mean_us"]), file=sys.stderr)
    if args.calibrate:
        ms, flop = hg.calibrate_mfma(20000, sh)
        buf = torch.ones(1 << 28, dtype=torch.int32, device="cuda")           # 1 GiB
        hg.calibrate_hbm_read(buf.data_ptr(), buf.numel() * 4, sh)            # warm-up (also fills no cache: 1 GiB > 256 MiB)
        ms_r = hg.calibrate_hbm_read(buf.data_ptr(), buf.numel() * 4, sh)
        cz = torch.empty((8192, 8192), dtype=torch.float16, device="cuda")
        with hg.Plan(8192, 8192, 0) as pz:                                    # K = 0: a pure 128 MiB fill of C
            pz.run(None, None, cz.data_ptr(), sh)
            torch.cuda.synchronize()
        out["calibration"] = {"mfma_only_tflops": flop / ms * 1e-9, "stream_read_gbs": buf.numel() * 4 / ms_r * 1e-6,
                              "read_kernel_bytes": buf.numel() * 4, "fill_kernel_bytes": 8192 * 8192 * 2}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    for s in sets:
        s["plan"].destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
