"""Cost model behind hgemm_plan()'s choice for shapes that are not in the dispatch table.

The paper's premise (Section 5, Section 6) is that the best kernel configuration depends on (M, N, K);
its Section 6 reads trends off the winners (tiles grow with M and N, stages with K, ...).  Here the
same idea is made executable: a small analytical model of one launch -- matrix-core time and
global->LDS copy time per K-tile, prologue / epilogue per workgroup, rounds of workgroups over 256
compute units, whole-problem memory time, the second pass of split-K -- whose ~30 constants are
fitted to measured times of every candidate configuration on random shapes.  hgemm_plan() evaluates
the model for each compiled configuration and split factor and takes the cheapest.

    python -m paper_2512_02551_amd.plan_model gather --seed 11 --shapes 300 --out FILE   # on the GPU
    python -m paper_2512_02551_amd.plan_model fit  [FILE ...]      # CPU; rewrites csrc/plan_model.inc
    python -m paper_2512_02551_amd.plan_model evaluate [FILE ...]  # CPU; regret of the model's choice

Timing files are JSON lines {"shape": [M, N, K], "cands": [[spec-without-family, microseconds], ...]};
csrc/plan_model_timings.jsonl.gz is the set the committed constants were fitted on.
predict_us() below and predict_us() in csrc/hgemm_api.hip are the same formula; a host test compares them.
"""
from __future__ import annotations

import argparse
import gzip
import json
import math
import os
import sys

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
DATA = os.path.join(_HERE, "csrc", "plan_model_timings.jsonl.gz")
INC = os.path.join(_HERE, "csrc", "plan_model.inc")

CUS = 256
LDS_PER_CU = 160 * 1024
CACHE_RESIDENT_BYTES = 192 * 2 ** 20      # below this the operands of back-to-back calls stay in the last-level cache

# name -> starting value.  Units: us, ns, bytes/ns (= GB/s) per compute unit, or plain factors.
PARAMS = {
    "T0": 1.7,        # launch floor, us
    "F": 13800.0,     # matrix-core rate of one compute unit, flop/ns
    "c1": 0.24,       # fragment-read overhead ~ (TM+TN)/(TM*TN)
    "q1": 1.14,       # factor for prefetch distance 1
    "m32": 1.2,       # factor for BM = 32
    "k128": 1.25,     # factor for BK = 128
    "k32": 0.95,      # factor for BK = 32
    "cp": 0.7,        # clock drop of long launches: factor 1 + cp * clip(log10(flop) - 10, 0, 2) / 2
    "BW": 200.0,      # global->LDS copy rate of one compute unit, bytes/ns
    "a2": 0.9, "a8": 1.75, "a16": 1.7,          # ... scaled by the number of waves (4 waves = 1)
    "b64": 0.75, "b256": 1.0,                   # ... and by BN (128 = 1)
    "L": 225.0,       # latency of a copy served by the L2, ns
    "Lh": 520.0,      # extra latency, times the share of the copied bytes that is first-touch data, problems larger than the last-level cache, ns
    "tk": 45.0,       # fixed cost per K-tile (barrier), ns
    "ov": 1.0,        # share of the shorter of {matrix-core, copy} time that does not overlap
    "Tpro": 0.5,      # prologue latency, us
    "e0": 0.35,       # epilogue fixed, us
    "BWepi": 68.0,    # epilogue store rate (fp16 tile), bytes/ns
    "BWp": 82.0,      # epilogue store rate (fp32 partial tile), bytes/ns
    "BWs": 16000.0,   # whole-chip read rate, cache-resident problems, GB/s
    "BWh": 3800.0,    # whole-chip read rate from HBM, GB/s
    "h64": 0.6, "h128": 0.85,                   # ... scaled by BN: a workgroup reads BN*2-byte pieces of B rows (256 = 1)
    "rr": 0.5,        # share of B that is fetched again by each further row of tiles (up to the 8 XCDs) when it does not stay cached
    "Lhb": 2500.0,    # HBM latency for the bytes-in-flight bound, ns
    "BWw1": 5400.0,   # rate at which the output (or the fp32 partials) drains when compute units hold one workgroup, GB/s
    "BWw2": 8300.0,   # ... two or more (stores of one workgroup overlap the main loop of another)
    "Tr0": 1.5,       # split-K second launch, us
    "Tr1": 1.0,       # ... per 8 splits, us
    "BWr": 5200.0,    # ... its traffic rate, GB/s
}
NAMES = list(PARAMS)


def parse_spec(spec: str) -> dict:
    d = {"tb": 0, "sm": 0, "gm": 8, "sk": 1, "pf": 1}
    for kv in spec.split(","):
        if "=" in kv:
            k, v = kv.split("=")
            d[k] = int(v)
    return d


def features(shape, s: dict) -> dict:
    """Integer features of one (shape, configuration); mirrored by plan_features() in hgemm_api.hip."""
    M, N, K = shape
    bm, bn, bk, wm, wn, st, pf, sk = s["bm"], s["bn"], s["bk"], s["wm"], s["wn"], s["st"], s["pf"], s["sk"]
    nw = wm * wn
    tiles = -(-M // bm) * -(-N // bn)
    kt = -(-K // bk)
    lds = st * (bm + bn) * bk * 2
    tm, tn = bm // wm // 32, bn // wn // 32
    regs = tm * tn * 16 + (pf + 1) * (tm + tn) * 4 + 40                 # accumulators + fragment sets + addressing
    wps = max(1, min(8, 512 // max(regs, 64)))                          # waves per SIMD the register file admits
    occ = max(1, min(LDS_PER_CU // lds, (wps * 4) // nw if nw <= wps * 4 else 1))
    return dict(M=M, N=N, K=K, bm=bm, bn=bn, bk=bk, nw=nw, st=st, pf=pf, sk=sk, tiles=tiles, kt=kt, tm=tm, tn=tn, occ=occ)


FEATURE_KEYS = ["M", "N", "K", "bm", "bn", "bk", "nw", "st", "pf", "sk", "tiles", "kt", "tm", "tn", "occ"]


def predict_us(g: dict, D: dict):
    """Predicted microseconds per call; g = constants by name, D = feature arrays (or scalars)."""
    M, N, K = D["M"], D["N"], D["K"]
    bm, bn, bk, sk, st, nw = D["bm"], D["bn"], D["bk"], D["sk"], D["st"], D["nw"]
    tiles, kt, occ, TM, TN = D["tiles"], D["kt"], D["occ"], D["tm"], D["tn"]
    wgs = tiles * sk
    kt_wg = np.ceil(kt / sk)
    w = np.ceil(wgs / CUS)                         # workgroups on the busiest compute unit
    co = np.minimum(occ, w)                        # ... of which this many are resident together
    rounds = np.ceil(w / co)
    flop = 2.0 * M * N * K
    big = np.clip(np.log10(np.maximum(flop, 1.0)) - 10.0, 0.0, 2.0) / 2.0
    t_mfma = 2.0 * bm * bn * bk / g["F"] * (1 + g["c1"] * (TM + TN) / (TM * TN)) * (1 + g["cp"] * big)
    t_mfma = t_mfma * np.where(D["pf"] == 1, g["q1"], 1.0) * np.where(bm == 32, g["m32"], 1.0)
    t_mfma = t_mfma * np.where(bk == 128, g["k128"], np.where(bk == 32, g["k32"], 1.0))
    stage = (bm + bn) * bk * 2.0
    bytes_in = 2.0 * (M * K + K * N)
    bytes_c = 2.0 * M * N
    part = np.where(sk > 1, sk * M * N * 4.0, 0.0)
    resident = (bytes_in + bytes_c) < CACHE_RESIDENT_BYTES
    miss = np.minimum(1.0, bytes_in / (wgs * kt_wg * stage))
    lat = g["L"] + miss * np.where(resident, 0.0, g["Lh"])
    peak = g["BW"] * np.where(nw == 2, g["a2"], np.where(nw == 8, g["a8"], np.where(nw == 16, g["a16"], 1.0)))
    peak = peak * np.where(bn == 64, g["b64"], np.where(bn == 256, g["b256"], 1.0))
    inflight = np.maximum(st - 1, 1) * stage * co
    bw = np.minimum(peak, inflight / lat) / co
    t_copy = stage / bw
    t_kt = np.maximum(t_mfma * co, t_copy) + g["ov"] * np.minimum(t_mfma * co, t_copy) + g["tk"]       # ns
    pro = g["Tpro"]
    epi = g["e0"] + np.where(sk > 1, bm * bn * 4.0 / g["BWp"], bm * bn * 2.0 / g["BWepi"]) * 1e-3
    cu_time = rounds * (kt_wg * t_kt * 1e-3 + pro + epi)
    tot_inflight = np.minimum(wgs, CUS * occ) * np.maximum(st - 1, 1) * stage
    bw_read = np.where(resident & (part + bytes_in + bytes_c < CACHE_RESIDENT_BYTES), g["BWs"],
                       np.minimum(g["BWh"] * np.where(bn == 64, g["h64"], np.where(bn == 128, g["h128"], 1.0)), tot_inflight / g["Lhb"]))
    writes = np.where(sk > 1, part, bytes_c)
    tiles_m = np.ceil(M / bm)
    hbm_bytes = np.where(resident, bytes_in, 2.0 * M * K + 2.0 * K * N * (1.0 + g["rr"] * (np.minimum(tiles_m, 8.0) - 1.0)))
    t_main = np.maximum(cu_time, hbm_bytes / bw_read * 1e-3) + writes / np.where(co <= 1, g["BWw1"], g["BWw2"]) * 1e-3
    t_red = np.where(sk > 1, g["Tr0"] + g["Tr1"] * np.ceil(sk / 8.0) + (part + bytes_c) / g["BWr"] * 1e-3, 0.0)
    return g["T0"] + t_main + t_red


def load_rows(paths):
    rows = []
    for p in paths:
        op = gzip.open if p.endswith(".gz") else open
        with op(p, "rt") as f:
            for line in f:
                if line.strip():
                    r = json.loads(line)
                    cands = []
                    for s, t in r["cands"]:
                        if s.startswith("mfma,"):
                            s = s[5:]
                        d = parse_spec(s)
                        if d["sm"] or d["tb"] or d["gm"] != 8:
                            continue
                        cands.append((s.replace(",gm=8", ""), float(t)))
                    best = float(r["best"]) if "best" in r else min(float(t) for _, t in r["cands"])
                    rows.append({"shape": r["shape"], "cands": cands, "best": best})
    return rows


def table(rows):
    feats, ts, ri = [], [], []
    for i, r in enumerate(rows):
        for s, t in r["cands"]:
            feats.append(features(r["shape"], parse_spec(s)))
            ts.append(t)
            ri.append(i)
    D = {k: np.array([f[k] for f in feats], dtype=np.float64) for k in FEATURE_KEYS}
    return D, np.array(ts), np.array(ri)


def regret(g, rows, D=None, ts=None, ri=None):
    """Per shape: measured time of the model's pick / best measured time of any candidate."""
    if D is None:
        D, ts, ri = table(rows)
    pred = predict_us(g, D)
    out = np.empty(len(rows))
    start = 0
    for i, r in enumerate(rows):
        n = len(r["cands"])
        out[i] = ts[start + int(np.argmin(pred[start:start + n]))] / r["best"]
        start += n
    return out


def read_inc(path=INC) -> dict:
    g = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line.startswith("PLAN_MODEL_CONST("):
                name, val = line[len("PLAN_MODEL_CONST("):].split(")")[0].split(",")
                g[name.strip()] = float(val)
    return g


def write_inc(g: dict, note: str, path=INC):
    with open(path, "w") as f:
        f.write("// Constants of the plan-time cost model (formula: predict_us() in hgemm_api.hip and in plan_model.py).\n"
                "// Written by `python -m paper_2512_02551_amd.plan_model fit`; do not edit by hand.\n"
                f"// {note}\n")
        for k in NAMES:
            f.write(f"PLAN_MODEL_CONST({k}, {g[k]:.9g})\n")


def fit(rows, verbose=True):
    from scipy.optimize import least_squares

    D, ts, ri = table(rows)
    p0 = np.log(np.array([PARAMS[k] for k in NAMES]))

    def resid(p):
        return np.log(predict_us(dict(zip(NAMES, np.exp(p))), D) / ts)

    best = None
    rs = np.random.default_rng(0)
    for trial in range(4):
        start = p0 + (rs.normal(0, 0.25, size=p0.shape) if trial else 0)
        r = least_squares(resid, start, loss="soft_l1", f_scale=0.2, max_nfev=400)
        g = dict(zip(NAMES, np.exp(r.x)))
        reg = regret(g, rows, D, ts, ri)
        score = math.exp(np.log(reg).mean())
        if verbose:
            print(f"start {trial}: rms log error {np.sqrt((resid(r.x) ** 2).mean()):.4f}, regret geomean {score:.4f}", flush=True)
        if best is None or score < best[0]:
            best = (score, g)
    return best[1]


def summarize(reg):
    return (f"geomean {math.exp(np.log(reg).mean()):.4f}, median {np.median(reg):.3f}, "
            f"90th percentile {np.quantile(reg, 0.9):.3f}, worst {reg.max():.3f} over {len(reg)} shapes")


def gather(seed: int, n_shapes: int, out: str):
    import random
    import time

    import torch

    import paper_2512_02551_amd as hg

    hg.load()
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    rng = random.Random(seed)

    def dim():
        return max(8, int(round(math.exp(rng.uniform(math.log(48), math.log(16384))) / 8)) * 8)

    def timed_eager(p, a, b, c, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            p.run(a.data_ptr(), b.data_ptr(), c.data_ptr(), sh)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    def measure(p, a, b, c, reps, graph):
        """Per-call microseconds, best of two batches.  Short problems are timed as replays of a captured graph of
        the batch: their kernels take less than the host needs per enqueue, which would flatten every difference."""
        if not graph:
            timed_eager(p, a, b, c, 2)
            return min(timed_eager(p, a, b, c, reps), timed_eager(p, a, b, c, reps))
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            cs = torch.cuda.current_stream().cuda_stream
            for _ in range(reps):
                p.run(a.data_ptr(), b.data_ptr(), c.data_ptr(), cs)
        g.replay()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(2):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            g.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) / reps * 1e3)
        return best

    t0 = time.time()
    done = 0
    with open(out, "w") as f:
        while done < n_shapes:
            M, N, K = dim(), dim(), dim()
            if M * N * K > 2 ** 37:
                continue
            a = (torch.rand(M, K, device="cuda") * 2 - 1).half()
            b = (torch.rand(K, N, device="cuda") * 2 - 1).half()
            c = torch.empty(M, N, device="cuda", dtype=torch.float16)
            graph = 2.0 * M * N * K < 2e10
            reps = 32 if graph else (16 if 2.0 * M * N * K < 3e10 else (6 if 2.0 * M * N * K < 3e11 else 3))
            with hg.Plan(M, N, K) as p:
                d = p.describe()
                t_def = measure(p, a, b, c, reps, graph)
            cands = []
            for spec in hg.candidates(M, N, K):
                try:
                    p = hg.Plan(M, N, K, None, spec)
                except hg.HgemmError:
                    continue
                cands.append((p.describe(), round(measure(p, a, b, c, reps, graph), 3)))
                p.destroy()
            f.write(json.dumps({"shape": [M, N, K], "default": [d, round(t_def, 3)], "graph_timed": graph, "cands": cands}) + "\n")
            f.flush()
            done += 1
            if done % 10 == 0:
                print(f"{done} shapes, {time.time() - t0:.0f} s", flush=True)


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    g_ = sub.add_parser("gather")
    g_.add_argument("--seed", type=int, default=11)
    g_.add_argument("--shapes", type=int, default=300)
    g_.add_argument("--out", required=True)
    f_ = sub.add_parser("fit")
    f_.add_argument("files", nargs="*", default=[DATA])
    e_ = sub.add_parser("evaluate")
    e_.add_argument("files", nargs="*", default=[DATA])
    args = ap.parse_args()
    if args.cmd == "gather":
        gather(args.seed, args.shapes, args.out)
    elif args.cmd == "fit":
        rows = load_rows(args.files)
        g = fit(rows)
        reg = regret(g, rows)
        write_inc(g, f"Fitted on {len(rows)} random shapes x all candidate configurations; regret of the model's pick: {summarize(reg)}.")
        print("wrote", INC, "--", summarize(reg))
    else:
        rows = load_rows(args.files)
        print(summarize(regret(read_inc(), rows)))


if __name__ == "__main__":
    sys.path.insert(0, os.path.dirname(_HERE))
    main()
