"""Summarises the measured dispatch table the way the paper analyses its 1,000 kernels (Section 6):
how the chosen tile sizes, stage counts, prefetch distance, split factors and tile order relate to
(M, N, K).  Reads csrc/dispatch_tuning_log.jsonl, prints Markdown.

    python -m paper_2512_02551_amd.analyze_dispatch
"""
from __future__ import annotations

import json
import math
import os
import re
from collections import Counter

_HERE = os.path.dirname(os.path.abspath(__file__))
LOG = os.path.join(_HERE, "csrc", "dispatch_tuning_log.jsonl")
PAPER_GRID = (64, 128, 256, 512, 1024, 2048, 4096, 8192, 12288, 16384)


def _spearman(x, y):
    def rank(v):
        order = sorted(range(len(v)), key=lambda i: v[i])
        r = [0.0] * len(v)
        i = 0
        while i < len(order):
            j = i
            while j + 1 < len(order) and v[order[j + 1]] == v[order[i]]:
                j += 1
            for k in range(i, j + 1):
                r[order[k]] = (i + j) / 2.0
            i = j + 1
        return r
    rx, ry = rank(x), rank(y)
    mx, my = sum(rx) / len(rx), sum(ry) / len(ry)
    num = sum((a - mx) * (b - my) for a, b in zip(rx, ry))
    den = math.sqrt(sum((a - mx) ** 2 for a in rx) * sum((b - my) ** 2 for b in ry))
    return num / den if den else float("nan")


def load(grid_only=True):
    rows = []
    with open(LOG) as f:
        for line in f:
            if not line.strip():
                continue
            r = json.loads(line)
            m, n, k = r["shape"]
            if grid_only and not all(v in PAPER_GRID for v in (m, n, k)):
                continue
            kv = dict(re.findall(r"(\w+)=(\d+)", r["spec"]))
            r["cfg"] = {key: int(val) for key, val in kv.items()}
            rows.append(r)
    return rows


def main():
    rows = load()
    print(f"Shapes analysed: {len(rows)} (the paper's grid {{64..16384}}^3 as far as it has been tuned)\n")
    M = [r["shape"][0] for r in rows]
    N = [r["shape"][1] for r in rows]
    K = [r["shape"][2] for r in rows]
    g = lambda key, d=0: [r["cfg"].get(key, d) for r in rows]
    print("| relation (Spearman rho) | this table (MI355X) | paper, Section 6 (A100) |")
    print("|---|---|---|")
    print(f"| BM vs M | {_spearman(g('bm'), M):.3f} | 0.652 |")
    print(f"| BN vs N | {_spearman(g('bn'), N):.3f} | 0.705 |")
    print(f"| BK vs K | {_spearman(g('bk'), K):.3f} | 0.256 |")
    print(f"| BM vs BN | {_spearman(g('bm'), g('bn')):.3f} | 0.695 |")
    print(f"| stages vs K | {_spearman(g('st'), K):.3f} | positive (2-3 stages for K <= 128, 6+ for K > 8K) |")
    print(f"| bytes in flight (stages-1)*(BM+BN)*BK*2 vs K | {_spearman([(c['st'] - 1) * (c['bm'] + c['bn']) * c['bk'] * 2 for c in (r['cfg'] for r in rows)], K):.3f} | - |")
    print(f"| split-K factor vs K / (M*N) | {_spearman(g('sk', 1), [k / (m * n) for m, n, k in zip(M, N, K)]):.3f} | (no split-K in the paper) |")
    print()

    # mean tile sizes by dimension
    print("| dimension value | mean BM at M = value | mean BN at N = value | mean BK at K = value | mean stages at K = value | share with split-K at K = value |")
    print("|---|---|---|---|---|---|")
    for v in PAPER_GRID:
        bm = [r["cfg"]["bm"] for r in rows if r["shape"][0] == v]
        bn = [r["cfg"]["bn"] for r in rows if r["shape"][1] == v]
        bk = [r["cfg"]["bk"] for r in rows if r["shape"][2] == v]
        st = [r["cfg"]["st"] for r in rows if r["shape"][2] == v]
        sk = [r["cfg"].get("sk", 1) > 1 for r in rows if r["shape"][2] == v]
        if not bm or not bn or not bk:
            continue
        print(f"| {v} | {sum(bm) / len(bm):.0f} | {sum(bn) / len(bn):.0f} | {sum(bk) / len(bk):.0f} | {sum(st) / len(st):.1f} | {100 * sum(sk) / len(sk):.0f} % |")
    print()

    # tile order by problem size (the paper's block-swizzle usage by M*N*K)
    print("| log2(M*N*K) | shapes | grouped tile order (gm > 0) chosen, among shapes with > 512 tiles (only there is the order tuned) | stream-K | prefetch distance 3 |")
    print("|---|---|---|---|---|")
    edges = [(0, 27), (27, 33), (33, 36), (36, 99)]
    for lo, hi in edges:
        sel = [r for r in rows if lo <= math.log2(r["shape"][0] * r["shape"][1] * r["shape"][2]) < hi]
        if not sel:
            continue
        many = [r for r in sel if math.ceil(r["shape"][0] / r["cfg"]["bm"]) * math.ceil(r["shape"][1] / r["cfg"]["bn"]) > 512]
        gm_many = sum(1 for r in many if r["cfg"].get("gm", 8) > 0)
        sm = sum(1 for r in sel if r["cfg"].get("sm", 0))
        pf = sum(1 for r in sel if r["cfg"].get("pf", 1) == 3)
        label = f"{lo}-{hi}" if hi < 99 else f">= {lo}"
        share_many = f"{100 * gm_many / len(many):.0f} % of {len(many)}" if many else "-"
        print(f"| {label} | {len(sel)} | {share_many} | {100 * sm / len(sel):.0f} % | {100 * pf / len(sel):.0f} % |")
    print()

    c = Counter((r["cfg"]["bm"], r["cfg"]["bn"], r["cfg"]["bk"], r["cfg"]["wm"] * r["cfg"]["wn"], r["cfg"]["st"], r["cfg"].get("pf", 1)) for r in rows)
    print("| most frequent (BM, BN, BK, waves, stages, PF) | shapes |")
    print("|---|---|")
    for cfg, cnt in c.most_common(10):
        print(f"| {cfg} | {cnt} |")
    print()
    tf = [r["tflops"] for r in rows]
    print(f"Geometric mean over these shapes: {math.exp(sum(math.log(t) for t in tf) / len(tf)):.1f} TFLOP/s; "
          f"arithmetic mean {sum(tf) / len(tf):.1f} TFLOP/s; best {max(tf):.1f} TFLOP/s.")


if __name__ == "__main__":
    main()
