"""CPU-only checks of the tooling around the library: the dispatch-table writer, the table itself,
the analysis script and bench.py's host-side pieces.  No kernel is launched."""
import json
import os
import re
import subprocess
import sys

import pytest

import paper_2512_02551_amd as hg
import workloads as wl
from paper_2512_02551_amd import tune

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_02551_amd", "csrc")


def test_table_writer_round_trip(tmp_path):
    log = tmp_path / "log.jsonl"
    rows = [{"shape": [64, 64, 64], "spec": "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=1,sk=1,gm=8", "median_us": 6.0, "tflops": 0.1, "gbs": 4.0},
            {"shape": [128, 64, 256], "spec": "mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=2,gm=8", "median_us": 7.0, "tflops": 0.6, "gbs": 16.0},
            {"shape": [64, 64, 64], "spec": "mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=1,gm=8", "median_us": 5.5, "tflops": 0.1, "gbs": 4.5}]
    log.write_text("\n".join(json.dumps(r) for r in rows) + "\n")
    table = tmp_path / "table.inc"
    assert tune.write_table(str(log), str(table)) == 2            # the later row for 64^3 replaces the earlier one
    text = table.read_text()
    assert '{64, 64, 64, "mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=1,gm=8"}' in text
    assert '{128, 64, 256, "mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=2,gm=8"}' in text
    assert text.count("{0, 0, 0,") == 1


@pytest.mark.parametrize("table,log", [("dispatch_table.inc", "dispatch_tuning_log.jsonl"), ("dispatch_table_tn.inc", "dispatch_tuning_log_tn.jsonl")])
def test_committed_table_names_only_compiled_kernels_and_covers_the_workloads(table, log):
    text = open(os.path.join(CSRC, table)).read()
    rows = re.findall(r'\{(\d+), (\d+), (\d+), "([^"]*)"\}', text)
    compiled = set()
    for line in hg.spec_help().splitlines():
        head = line.strip()
        # the deep-staged configurations and those on the 16 x 16 x 32 instruction have lines of their own
        if "compiled" in line or head.startswith("deep (bm") or head.startswith("mi16 (bm"):
            for tup in line.split(":")[1].split():
                compiled.add(tuple(int(x) for x in tup.strip("()").split(",")) + (16 if head.startswith("mi16") else 32,))
    shapes = set()
    for m, n, k, spec in rows:
        if not spec:
            continue
        shapes.add((int(m), int(n), int(k)))
        if spec.startswith("skinny,"):          # the streaming family: one kernel template, no tile configuration to look up
            assert int(m) <= 64 and re.fullmatch(r"skinny,sk=\d+(,fr=1)?(,wv=(8|16))?", spec), spec
            continue
        kv = dict(re.findall(r"(\w+)=(\d+)", spec))
        key = tuple(int(kv.get(x, 1 if x == "pf" else 0)) for x in ("bm", "bn", "bk", "wm", "wn", "st", "pf")) + (int(kv.get("mi", 32)),)
        assert key in compiled, f"table row {m}x{n}x{k} names a kernel that is not compiled: {spec}"
        if table.endswith("_tn.inc"):          # column-major B: no transposing copy, and 64-byte K runs (bk = 32) never win
            assert "tb=1" not in spec
    for s in [wl.C1_SHAPE, *wl.C2_SHAPES, *wl.C3_SHAPES, *wl.c4_shapes(), *wl.C5_SHAPES, wl.C5_INT_SHAPE]:
        assert s in shapes, f"workload shape {s} has no table row"
    assert set(wl.C3_LARGE_SHAPES) <= shapes and set(wl.C3_OTHER_SHAPES) <= shapes
    # the table and the log it was written from agree
    log_shapes = {tuple(json.loads(l)["shape"]) for l in open(os.path.join(CSRC, log)) if l.strip()}
    assert log_shapes == shapes


def test_tuner_shape_lists():
    assert len(tune.all_shapes(["P"])) == 1000
    assert set(wl.c4_shapes()) <= set(tune.all_shapes(["P"]))
    assert len(tune.all_shapes(["C1", "C2", "C3", "C4", "C5"])) == 1 + 4 + 20 + 200 + 3 - 4     # C2 ⊂ ... four C4 shapes repeat C2/C3


def test_analysis_script_runs():
    out = subprocess.run([sys.executable, "-m", "paper_2512_02551_amd.analyze_dispatch"], cwd=ROOT, capture_output=True, text=True, check=True).stdout
    assert "BM vs M" in out and "Geometric mean" in out


def test_bench_refuses_more_than_one_gpu():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in res.stderr


def test_bench_workload_tables():
    import bench
    for name, count in (("C1", 1), ("C2", 4), ("C3", 20), ("C4", 200), ("C5", 2)):
        shapes, gen = bench.workload_shapes(name)
        assert len(shapes) == count
    assert bench.PEAK_FP16_TFLOPS == 2500.0 and bench.PEAK_HBM_GBS == 8000.0


def test_bench_defaults_and_profiled_traffic_cover_the_roofline_shapes(monkeypatch):
    """The default run sorts a step's shapes by work, and every shape that can become `roofline` (the largest
    compute-bound one) or `roofline_hbm` (the memory-bound skinny ones with M <= 16) has a profiled traffic figure
    at least as large as its algorithmic bytes."""
    import bench
    import workloads as wl
    monkeypatch.setattr(sys, "argv", ["bench.py"])
    args = bench.parse_args()
    assert args.order == "flop" and args.gpus == 1
    need = [max(wl.C5_SHAPES, key=lambda s: s[0] * s[1] * s[2])] + [s for s in wl.C3_SHAPES if s[0] <= 16]
    for (M, N, K) in need:
        assert (M, N, K) in bench.PROFILED_TRAFFIC_BYTES, (M, N, K)
        assert bench.PROFILED_TRAFFIC_BYTES[(M, N, K)] >= 2.0 * (M * K + K * N + M * N) * 0.98
