"""Autotuner: fills csrc/dispatch_table.inc with the fastest specialisation per (M,N,K).

    python -m paper_2512_02551_amd.tune [--workloads C1,C2,C3,C4,C5,P] [--out-log FILE] [--resume]

Protocol (after the library-autotuning procedure the paper describes in Section 2.2.3 and
its appendix: enumerate candidates, time each with warm-up rounds and a shuffled order per
round, keep the best median):
  1. candidates come from hgemm_candidates() (tile sizes, stages, split-K factors, tile order);
  2. every candidate must first reproduce, bit for bit, the generic kernel's result on
     small-integer inputs of the same shape (exact in fp32, so any summation order agrees);
     the largest shapes are compared on three bands of rows, the rest in full;
  3. a coarse pass times all survivors, a fine pass re-times the best few with more rounds; one sample
     is the per-call time of a batch of back-to-back calls between one pair of events (for problems
     below 2e10 flop the batch is captured in a graph and replayed, so that GPU time is compared and
     not the host's enqueue rate);
  4. the winner and its numbers are appended to a log (so a sweep can resume) and the table is
     rewritten from the log.
Inputs are drawn on the device; only timing and bitwise comparison happen here, all arithmetic
runs in the library's kernels.
"""
from __future__ import annotations

import argparse
import json
import os
import random
import re
import sys
import time

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
TABLE = os.path.join(_HERE, "csrc", "dispatch_table.inc")
DEFAULT_LOG = os.path.join(_HERE, "csrc", "dispatch_tuning_log.jsonl")
# B column-major (the TN layout of Section 2.2.2): a table of its own, for the shapes tuned in that layout
TABLE_TN = os.path.join(_HERE, "csrc", "dispatch_table_tn.inc")
DEFAULT_LOG_TN = os.path.join(_HERE, "csrc", "dispatch_tuning_log_tn.jsonl")


def all_shapes(workloads):
    sys.path.insert(0, os.path.dirname(_HERE))
    import workloads as wl

    out = []
    if "C1" in workloads:
        out.append(wl.C1_SHAPE)
    if "C2" in workloads:
        out += list(wl.C2_SHAPES)
    if "C3" in workloads:
        out += list(wl.C3_SHAPES)
    if "C3L" in workloads:     # LLM projections of a larger model (beyond the five configurations)
        out += list(wl.C3_LARGE_SHAPES)
    if "C3O" in workloads:     # LLM projections of other model widths (beyond the five configurations)
        out += list(wl.C3_OTHER_SHAPES)
    if "C4" in workloads:
        out += wl.c4_shapes()
    if "C5" in workloads:
        out += list(wl.C5_SHAPES) + [wl.C5_INT_SHAPE]
    if "P" in workloads:       # the paper's full grid: all 10^3 triples over {64, ..., 16384} (Abstract)
        v = wl.PAPER_GRID_VALUES
        out += [(m, n, k) for m in v for n in v for k in v]
    seen, uniq = set(), []
    for s in out:
        if s not in seen:
            seen.add(s)
            uniq.append(s)
    return uniq


def write_table(log_path: str, table_path: str = TABLE) -> int:
    tn = os.path.basename(table_path) == os.path.basename(TABLE_TN)
    rows = {}
    if os.path.exists(log_path):
        with open(log_path) as f:
            for line in f:
                line = line.strip()
                if line:
                    r = json.loads(line)
                    rows[tuple(r["shape"])] = r
    with open(table_path, "w") as f:
        if tn:
            f.write("// Per-shape dispatch table for column-major B (the TN layout): same form as dispatch_table.inc, filled by\n"
                    "// python -m paper_2512_02551_amd.tune --layout tn.  Shapes it does not hold use the row of the NN table.\n"
                    "static const DispatchRow kDispatchTableTN[] = {\n"
                    "    {0, 0, 0, \"\"},\n")
        else:
            f.write("// Per-shape dispatch table: (M, N, K) -> specialisation, filled from timed runs on one MI355X\n"
                    "// by the autotuner (python -m paper_2512_02551_amd.tune).  An empty spec means \"use the cost model\".\n"
                    "// Columns of the trailing comment: median microseconds, TFLOP/s, GB/s of algorithmic traffic.\n"
                    "struct DispatchRow { int64_t m, n, k; const char* spec; };\n"
                    "static const DispatchRow kDispatchTable[] = {\n"
                    "    {0, 0, 0, \"\"},\n")
        for (m, n, k) in sorted(rows):
            r = rows[(m, n, k)]
            f.write(f"    {{{m}, {n}, {k}, \"{r['spec']}\"}},  // {r['median_us']:.1f} us, {r['tflops']:.1f} TFLOP/s, {r['gbs']:.0f} GB/s\n")
        f.write("};\n")
    return len(rows)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workloads", default="C1,C2,C3,C4,C5")
    ap.add_argument("--layout", choices=["nn", "tn"], default="nn",
                    help="tn: B column-major (stored N x K); candidates, gate and timing use that layout and the result goes "
                         "to the TN log and table")
    ap.add_argument("--out-log", default="", help="default: the committed log of the layout")
    ap.add_argument("--resume", action="store_true")
    ap.add_argument("--coarse", type=int, default=7)
    ap.add_argument("--fine", type=int, default=30)
    ap.add_argument("--top", type=int, default=4)
    ap.add_argument("--table-only", action="store_true")
    ap.add_argument("--combine", default="",
                    help="comma-separated refinement logs (made with --candidates-from): combine them into --out-log and "
                         "rewrite the table; no GPU work")
    ap.add_argument("--max-shapes", type=int, default=0)
    ap.add_argument("--max-k", type=int, default=0, help="only shapes with K <= this (re-tuning a slice of a workload)")
    ap.add_argument("--shapes", default="", help="further shapes MxNxK,MxNxK,... tuned after the workloads' (use --workloads '' for these "
                                                 "alone); those with fewer than 312 flop per byte of operands are timed with rotating operand sets")
    ap.add_argument("--max-m", type=int, default=0, help="only shapes with M <= this (e.g. the shapes the skinny family can run)")
    ap.add_argument("--max-flop", type=float, default=0.0, help="only shapes with 2*M*N*K <= this")
    ap.add_argument("--min-flop", type=float, default=0.0, help="only shapes with 2*M*N*K >= this")
    ap.add_argument("--graph-below-flop", type=float, default=2e10,
                    help="shapes with 2*M*N*K below this are timed as replays of a captured graph of the batch: their "
                         "kernels are shorter than the host's enqueue time, which would otherwise hide every difference")
    ap.add_argument("--candidates-from", default="",
                    help="comma-separated tuning logs: instead of every candidate, time only the specs these logs record "
                         "for the shape (winners and runners-up) -- a refinement pass that settles close calls between "
                         "earlier sweeps with many more rounds per candidate")
    ap.add_argument("--fused-twins", action="store_true",
                    help="with --candidates-from: also time, for every recorded split-K spec, its twin with the reduction "
                         "fused into the kernel (fr=1), and tune only the shapes that have a split-K spec on record")
    ap.add_argument("--extra-specs", default="",
                    help="with --candidates-from: ';'-separated specs timed on top of the recorded ones (a new "
                         "configuration tried on the shapes where a given kind of spec is on record)")
    ap.add_argument("--only-recorded-with", default="",
                    help="with --candidates-from: tune only the shapes that have a spec containing this text on record")
    ap.add_argument("--merge-into", default="", help="after tuning, replace the rows of these shapes in this log and rewrite the table from it")
    ap.add_argument("--cold-workloads", default="C3,C3L,C3O",
                    help="workloads whose shapes are timed with rotating operand sets (> 768 MiB between reuses), "
                         "so that the choice is made for data coming from HBM, not from the last-level cache")
    args = ap.parse_args()
    tn = args.layout == "tn"
    table = TABLE_TN if tn else TABLE
    if not args.out_log:
        args.out_log = DEFAULT_LOG_TN if tn else DEFAULT_LOG

    if args.combine:
        print("rows changed:", combine_passes([p for p in args.combine.split(",") if p], args.out_log))
        print("rows:", write_table(args.out_log, table))
        return
    if args.table_only:
        print("rows:", write_table(args.out_log, table))
        return

    import torch

    import paper_2512_02551_amd as hg

    hg.load()
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    lay = hg.Layouts.make(b_col_major=True) if tn else None

    done = set()
    if args.resume and os.path.exists(args.out_log):
        with open(args.out_log) as f:
            for line in f:
                if line.strip():
                    done.add(tuple(json.loads(line)["shape"]))
    elif os.path.exists(args.out_log):
        os.remove(args.out_log)

    extra = [tuple(int(v) for v in item.split("x")) for item in args.shapes.split(",") if item]
    shapes = [s for s in all_shapes(args.workloads.split(",")) + [e for e in extra if e not in all_shapes(args.workloads.split(","))] if s not in done]
    cold_shapes = set(all_shapes([w for w in args.cold_workloads.split(",") if w])) if args.cold_workloads else set()
    cold_shapes |= {(m, n, k) for (m, n, k) in extra if m * n * k / (m * k + k * n + m * n) < 312}
    if args.max_k:
        shapes = [s for s in shapes if s[2] <= args.max_k]
    if args.max_m:
        shapes = [s for s in shapes if s[0] <= args.max_m]
    if args.max_flop:
        shapes = [s for s in shapes if 2.0 * s[0] * s[1] * s[2] <= args.max_flop]
    if args.min_flop:
        shapes = [s for s in shapes if 2.0 * s[0] * s[1] * s[2] >= args.min_flop]
    if args.max_shapes:
        shapes = shapes[:args.max_shapes]
    rng = random.Random(0)
    t_start = time.time()
    recorded = {}
    for path in [p for p in args.candidates_from.split(",") if p]:
        with open(path) as f:
            for line in f:
                if line.strip():
                    r = json.loads(line)
                    specs = recorded.setdefault(tuple(r["shape"]), [])
                    for sp in [r["spec"]] + [x[0] for x in r.get("runner_up", [])]:
                        sp = sp.replace(",pad=1", "")
                        if sp and sp not in specs:
                            specs.append(sp)
    if args.only_recorded_with:
        recorded = {k: v for k, v in recorded.items() if any(args.only_recorded_with in sp for sp in v)}
        shapes = [s for s in shapes if s in recorded]
    for specs in recorded.values():
        specs += [sp for sp in args.extra_specs.split(";") if sp and sp not in specs]
    if args.fused_twins:
        def splits(sp):
            m = re.search(r"sk=(\d+)", sp)
            return int(m.group(1)) if m else 1
        recorded = {k: v for k, v in recorded.items() if any(splits(sp) > 1 for sp in v)}
        for specs in recorded.values():
            for sp in list(specs):
                if splits(sp) > 1 and "fr=1" not in sp and "sm=1" not in sp and sp + ",fr=1" not in specs:
                    specs.append(sp + ",fr=1")
        shapes = [s for s in shapes if s in recorded]

    rot = {"sets": None, "i": 0, "graph": False, "graphs": {}}
    hgemm_run = hg.load().hgemm_run          # bound once: the eager batches should cost the host as little as Python allows

    def timed(plan, a, b, c, rounds):
        """One sample: `rounds` back-to-back calls between one pair of events, per-call time.  With
        rot["graph"] the batch is captured once per (plan, rounds) and the sample is one replay."""
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        if rot["graph"] and rot["sets"] is None:
            key = (id(plan), rounds)
            g = rot["graphs"].get(key)
            if g is None:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    cs = torch.cuda.current_stream().cuda_stream
                    for r in range(rounds):
                        plan.run(a.data_ptr(), b.data_ptr(), c.data_ptr(), cs)
                rot["graphs"][key] = g
                g.replay()
                torch.cuda.synchronize()
            e0.record(stream)
            g.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            return [e0.elapsed_time(e1) / rounds]
        h = plan._h
        if rot["sets"] is not None:
            ptrs = [rot["ptrs"][(rot["i"] + r) % len(rot["ptrs"])] for r in range(rounds)]
            rot["i"] += rounds
        else:
            ptrs = [(a.data_ptr(), b.data_ptr(), c.data_ptr())] * rounds
        e0.record(stream)
        for (pa, pb, pc) in ptrs:
            if hgemm_run(h, pa, pb, pc, sh):
                raise RuntimeError("hgemm_run failed")
        e1.record(stream)
        torch.cuda.synchronize()
        return [e0.elapsed_time(e1) / rounds]

    for idx, (M, N, K) in enumerate(shapes):
        gen = torch.Generator(device="cuda")
        gen.manual_seed(M * 1000003 + N * 1009 + K)
        # timing inputs: uniform[-1,1]; gate inputs: integers in {-2..2}
        a = (torch.rand((M, K), device="cuda", generator=gen) * 2 - 1).half()
        b = (torch.rand((K, N), device="cuda", generator=gen) * 2 - 1).half()
        ai = torch.randint(-2, 3, (M, K), device="cuda", generator=gen).half()
        bi = torch.randint(-2, 3, (K, N), device="cuda", generator=gen).half()
        if tn:                                    # the same matrices, stored N x K
            b, bi = b.t().contiguous(), bi.t().contiguous()
        c = torch.empty((M, N), device="cuda", dtype=torch.float16)
        cref = torch.empty((M, N), device="cuda", dtype=torch.float16)
        rot["sets"] = None
        if (M, N, K) in cold_shapes:
            per_set = 2 * (M * K + K * N + M * N)
            n_sets = max(2, min(64, -(-768 * 2 ** 20 // per_set)))
            rot["sets"] = [(a, b, c)] + [(a.clone(), b.clone(), torch.empty_like(c)) for _ in range(n_sets - 1)]
            rot["ptrs"] = [(x.data_ptr(), y.data_ptr(), z.data_ptr()) for (x, y, z) in rot["sets"]]
        rot["graph"] = rot["sets"] is None and 2.0 * M * N * K < args.graph_below_flop
        rot["graphs"] = {}
        # The gate: the generic kernel's result on the integer inputs.  Above 2^37 multiply-adds the
        # one-thread-per-element kernel would take seconds, so there it computes three bands of 16 rows
        # (first, middle, last) and every candidate is compared on those rows only.
        full_gate = M * N * K <= 2 ** 37
        bands = []
        if full_gate:
            with hg.Plan(M, N, K, lay, "generic") as p:
                p.run(ai.data_ptr(), bi.data_ptr(), cref.data_ptr(), sh)
                torch.cuda.synchronize()
        else:
            for r0 in sorted({0, (M // 2) // 16 * 16, max(0, M - 16)}):
                rows = min(16, M - r0)
                band = torch.empty((rows, N), device="cuda", dtype=torch.float16)
                with hg.Plan(rows, N, K, lay, "generic") as p:
                    p.run(ai[r0:r0 + rows].data_ptr(), bi.data_ptr(), band.data_ptr(), sh)
                    torch.cuda.synchronize()
                bands.append((r0, rows, band))
        plans = []
        rejected = 0
        for spec in (recorded.get((M, N, K)) or hg.candidates(M, N, K, lay)):
            try:
                p = hg.Plan(M, N, K, lay, spec)
            except hg.HgemmError:
                continue
            c.fill_(float("nan"))
            p.run(ai.data_ptr(), bi.data_ptr(), c.data_ptr(), sh)
            torch.cuda.synchronize()
            pairs = [(c, cref)] if full_gate else [(c[r0:r0 + rows], band) for (r0, rows, band) in bands]
            ok = True
            for got, want in pairs:
                if not torch.equal(got.view(torch.int16), want.view(torch.int16)):
                    # integer results can differ from the fp16-rounded generic result only through
                    # rounding of |C| > 2048; compare in fp32-exact territory only
                    small = want.abs() <= 2048
                    if not torch.equal(got[small], want[small]):
                        ok = False
            if not ok:
                rejected += 1
                p.destroy()
                continue
            plans.append([p.describe(), p, []])
        if not plans:
            print(f"[{idx + 1}/{len(shapes)}] {M}x{N}x{K}: no candidate", flush=True)
            continue
        # coarse pass, shuffled order per round group
        for entry in plans:
            if not rot["graph"]:                      # a graph's first (untimed) replay is its warm-up
                timed(entry[1], a, b, c, 2 if 2.0 * M * N * K < 2e12 else 1)
        order = list(range(len(plans)))
        rng.shuffle(order)
        coarse = args.coarse if 2.0 * M * N * K < 2e12 else max(2, args.coarse // 3)
        fine = max(1, args.fine // 3)
        if rot["graph"]:                              # replays are cheap and the kernels short: longer batches
            coarse, fine = 3 * coarse, 3 * fine
        for i in order:
            plans[i][2] += timed(plans[i][1], a, b, c, coarse)
        plans.sort(key=lambda e: float(np.median(e[2])))
        best = plans[:args.top]
        for entry in best:
            entry[2] = []
        for _ in range(3):
            order = list(range(len(best)))
            rng.shuffle(order)
            for i in order:
                best[i][2] += timed(best[i][1], a, b, c, fine)
        best.sort(key=lambda e: float(np.median(e[2])))
        spec, _, ts = best[0]
        med = float(np.median(ts))
        row = {"shape": [M, N, K], "spec": spec, "median_us": med * 1e3, "min_us": float(min(ts)) * 1e3,
               "tflops": 2.0 * M * N * K / med * 1e-9, "gbs": 2.0 * (M * K + K * N + M * N) / med * 1e-6,
               "candidates": len(plans), "rejected": rejected, "gated": "full" if full_gate else "row bands", "cold": rot["sets"] is not None,
               "graph_timed": bool(rot["graph"]),
               "runner_up": [(e[0], float(np.median(e[2])) * 1e3) for e in best[1:3]]}
        if recorded.get((M, N, K)):          # refinement pass: keep every candidate's time, passes on several boxes can then be combined
            row["all"] = [(e[0], float(np.median(e[2])) * 1e3) for e in best]
        with open(args.out_log, "a") as f:
            f.write(json.dumps(row) + "\n")
        print(f"[{idx + 1}/{len(shapes)}] {M}x{N}x{K}: {spec}  {row['median_us']:.1f} us  {row['tflops']:.1f} TFLOP/s  "
              f"{row['gbs']:.0f} GB/s  ({len(plans)} candidates, {rejected} rejected, {time.time() - t_start:.0f} s)", flush=True)
        rot["graphs"] = {}
        for entry in plans:
            entry[1].destroy()
        rot["sets"] = None
        del a, b, ai, bi, c, cref
    if args.merge_into:
        merge_logs(args.merge_into, args.out_log)
        print("rows:", write_table(args.merge_into, table), flush=True)
    else:
        print("rows:", write_table(args.out_log, table), flush=True)


def combine_passes(paths, main_log: str) -> int:
    """Combine refinement passes (logs whose rows carry every candidate's time, e.g. runs on several boxes): per
    shape, the spec with the smallest median, over the passes, of time / that pass's best time; its row in
    main_log is replaced (median time over the passes)."""
    import statistics

    def read(path):
        with open(path) as f:
            return {tuple(r["shape"]): r for r in (json.loads(line) for line in f if line.strip())}
    passes = [read(p) for p in paths]
    rows = []
    if os.path.exists(main_log):
        with open(main_log) as f:
            rows = [json.loads(line) for line in f if line.strip()]
    known = {tuple(r["shape"]) for r in rows}
    rows += [passes[0][s] for s in passes[0] if s not in known]
    changed = 0
    for i, r in enumerate(rows):
        s = tuple(r["shape"])
        if not all(s in p and p[s].get("all") for p in passes):
            continue
        score = {}
        for p in passes:
            best = min(t for _, t in p[s]["all"])
            for sp, t in p[s]["all"]:
                score.setdefault(sp, []).append(t / best)
        cand = {sp: statistics.median(v) for sp, v in score.items() if len(v) == len(passes)}
        if not cand:
            continue
        sp = min(cand, key=cand.get)
        times = lambda x: [t for p in passes for (y, t) in p[s]["all"] if y == x]
        med = statistics.median(times(sp))
        M, N, K = s
        new = dict(passes[0][s])
        new.pop("all", None)
        new.update({"spec": sp, "median_us": med, "min_us": min(times(sp)), "tflops": 2.0 * M * N * K / med * 1e-6,
                    "gbs": 2.0 * (M * K + K * N + M * N) / med * 1e-3, "passes": len(passes),
                    "runner_up": sorted([(x, statistics.median(times(x))) for x in cand if x != sp], key=lambda z: z[1])[:2]})
        changed += new["spec"] != r.get("spec")
        rows[i] = new
    with open(main_log, "w") as f:
        for r in rows:
            f.write(json.dumps(r) + "\n")
    return changed


def merge_logs(main_log: str, new_log: str) -> None:
    """Rows of new_log replace the rows of the same shapes in main_log (file order otherwise kept)."""
    def read(path):
        out = []
        if os.path.exists(path):
            with open(path) as f:
                out = [json.loads(line) for line in f if line.strip()]
        return out
    new = {tuple(r["shape"]): r for r in read(new_log)}
    rows = [new.pop(tuple(r["shape"]), r) for r in read(main_log)] + list(new.values())
    with open(main_log, "w") as f:
        for r in rows:
            f.write(json.dumps(r) + "\n")


if __name__ == "__main__":
    main()
