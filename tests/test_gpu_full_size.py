"""GPU parity at the benchmark's full sizes, with the plans bench.py times (dispatch table / cost model):
sampled outputs evaluated one by one by the oracle, and full comparison where the oracle finishes in seconds."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2512_02551_amd as hg  # noqa: E402
import workloads as wl  # noqa: E402
from oracle import hgemm_oracle as orc  # noqa: E402

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import TOL, assert_bit_exact, assert_close, run_hgemm  # noqa: E402


def _check_sampled(a, b, c, count, what):
    ii, jj = wl.sample_positions((a.shape[0], b.shape[1], a.shape[1]), count)
    ref = orc.hgemm_at(a, b, ii, jj).astype(np.float64)
    got = c[ii, jj].astype(np.float64)
    assert not np.isnan(got).any(), what
    err = np.abs(got - ref)
    bound = TOL * np.maximum(1.0, np.abs(ref))
    assert (err <= bound).all(), f"{what}: worst {float((err / bound).max()):.3g}x the bound"
    return float((err / bound).max())


def test_c1_single_256_cubed_full():
    a, b = wl.c1_inputs()
    c, _, _, desc = run_hgemm(a, b)
    assert_close(c, orc.hgemm(a, b), "C1 " + desc)


@pytest.mark.parametrize("shape", wl.C2_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_c2_square_sweep(shape):
    a, b = wl.c2_inputs(shape)
    c, _, _, desc = run_hgemm(a, b)
    if shape[0] <= 1024:
        assert_close(c, orc.hgemm(a, b), f"C2 {shape} {desc}")
    else:
        worst = _check_sampled(a, b, c, 4000, f"C2 {shape} {desc}")
        print(f"C2 {shape} [{desc}] worst error {worst:.3g} of the bound")


@pytest.mark.parametrize("shape", wl.C3_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_c3_llm_skinny_shapes(shape):
    a, b = wl.c3_inputs(shape)
    c, before, after, desc = run_hgemm(a, b, guard=1)
    _check_sampled(a, b, c, 3000, f"C3 {shape} {desc}")
    assert np.isnan(before).all() and np.isnan(after).all()


def test_c3_small_m_full_rows():
    # M = 1 and M = 16 against the full oracle product on a narrower N (the oracle's cost is M*N*K)
    for shape in [(1, 4096, 4096), (16, 4096, 4096)]:
        a, b = wl.c3_inputs(shape)
        c, _, _, desc = run_hgemm(a, b)
        assert_close(c, orc.hgemm(a, b), f"C3 {shape} {desc}")


@pytest.mark.parametrize("shape", wl.c4_shapes(), ids=lambda s: "x".join(map(str, s)))
def test_c4_grid_shapes(shape):
    """Every one of the 200 grid shapes with the plan the benchmark times: real inputs at sampled positions
    within the tolerance, then the exact-integer family of the same shape bit for bit at sampled positions."""
    a, b = wl.c4_inputs(shape)
    c, _, _, desc = run_hgemm(a, b)
    _check_sampled(a, b, c, 1500, f"C4 {shape} {desc}")
    del a, b, c
    name, ai, bi = wl.exact_family_for(shape, seed=11)
    ci, _, _, _ = run_hgemm(ai, bi)
    ii, jj = wl.sample_positions(shape, 1500, seed=1)
    ref = orc.hgemm_at(ai, bi, ii, jj)
    got = ci[ii, jj]
    sel = np.abs(ref.astype(np.float64)) <= 2048
    assert sel.mean() > 0.5
    assert np.array_equal(got[sel].astype(np.float64), ref[sel].astype(np.float64)), f"{shape} {name} {desc}"


def test_c5_small_integer_16384_full_bit_exact():
    shape = wl.C5_INT_SHAPE
    a, b = wl.small_int_inputs(shape, seed=0)
    ref = orc.hgemm(a, b)                      # 3.4e10 multiply-adds, seconds on the machine's cores
    c, _, _, desc = run_hgemm(a, b)
    assert np.abs(ref.astype(np.float64)).max() <= 2048
    assert_bit_exact(c, ref, f"C5 integer {desc}")


@pytest.mark.parametrize("shape", wl.C5_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_c5_large_16384_sampled(shape):
    a, b = wl.c5_inputs(shape)
    c, _, _, desc = run_hgemm(a, b)
    worst = _check_sampled(a, b, c, 4000, f"C5 {shape} {desc}")
    print(f"C5 {shape} [{desc}] worst error {worst:.3g} of the bound")
    del a, b, c
    # the paper's exactness criterion (Section 2.3.2) at the same size: {0,1} inputs, every sampled
    # position whose exact value is at most 2048 must match bit for bit
    name, ai, bi = wl.exact_family_for(shape, seed=13)
    ci, _, _, _ = run_hgemm(ai, bi)
    ii, jj = wl.sample_positions(shape, 4000, seed=3)
    ref = orc.hgemm_at(ai, bi, ii, jj)
    sel = np.abs(ref.astype(np.float64)) <= 2048
    assert sel.mean() > 0.5, name
    assert np.array_equal(ci[ii, jj][sel].astype(np.float64), ref[sel].astype(np.float64)), f"C5 {shape} {name} {desc}"


@pytest.mark.parametrize("shape", [(520, 1032, 776), (72, 4104, 1016), (3000, 5000, 136), (24, 8200, 2056), (1, 1000, 12296),
                                   (4100, 264, 4104), (8, 8, 16392), (2056, 2056, 2056), (6000, 6008, 520)],
                         ids=lambda s: "x".join(map(str, s)))
def test_shapes_outside_the_table_use_the_cost_model(shape):
    """Shapes the dispatch table does not hold (ragged tiles in every dimension): planned by the
    cost model, checked on sampled positions with real inputs and bit for bit with exact integers."""
    M, N, K = shape
    with hg.Plan(M, N, K) as p:
        chosen = p.describe()
    def deep_staged(s):                                    # pf longer than a K-tile: timed by the tuner, never chosen by the model
        f = dict(kv.split("=") for kv in s.split(",")[1:])
        return s.startswith("mfma") and int(f["pf"]) > int(f["bk"]) // 16

    cands = [s for s in hg.candidates(M, N, K) if "sm=1" not in s and "tb=1" not in s and "ps=1" not in s and ("gm=8" in s or s.startswith("skinny"))
             and ("fr=1" not in s or s.startswith("skinny")) and not deep_staged(s)]
    assert not deep_staged(chosen), chosen
    assert hg.predict_us(M, N, K, chosen) <= min(hg.predict_us(M, N, K, s) for s in cands) * (1 + 1e-12), chosen
    rng = np.random.default_rng([M, N, K])
    a = wl.uniform_pm1(rng, M, K)
    b = wl.uniform_pm1(rng, K, N)
    c, before, after, desc = run_hgemm(a, b, guard=1)
    assert desc.startswith(("mfma", "skinny")), desc
    _check_sampled(a, b, c, 2500, f"{shape} {desc}")
    assert np.isnan(before).all() and np.isnan(after).all()
    name, ai, bi = wl.exact_family_for(shape, seed=3)
    ci, _, _, _ = run_hgemm(ai, bi)
    ii, jj = wl.sample_positions(shape, 2500, seed=2)
    ref = orc.hgemm_at(ai, bi, ii, jj)
    sel = np.abs(ref.astype(np.float64)) <= 2048
    assert np.array_equal(ci[ii, jj][sel].astype(np.float64), ref[sel].astype(np.float64)), f"{shape} {name} {desc}"


@pytest.mark.parametrize("shape", [(65536, 8, 8), (8, 65536, 8), (8, 8, 65536), (1, 8, 262144), (200000, 16, 16), (3, 100000, 40),
                                   (1, 1000003, 8), (50000, 24, 4104)], ids=lambda s: "x".join(map(str, s)))
def test_extreme_aspect_ratios(shape):
    """One dimension far larger than the others (well outside the tuned table and the cost model's fitting range):
    whatever the planner picks must still be exact on integer inputs at sampled positions and stay inside C."""
    M, N, K = shape
    name, a, b = wl.exact_family_for(shape, seed=21)
    c, before, after, desc = run_hgemm(a, b, guard=1)
    ii, jj = wl.sample_positions(shape, 4000, seed=4)
    ref = orc.hgemm_at(a, b, ii, jj)
    sel = np.abs(ref.astype(np.float64)) <= 2048
    assert sel.mean() > 0.5, name
    assert np.array_equal(c[ii, jj][sel].astype(np.float64), ref[sel].astype(np.float64)), f"{shape} {name} {desc}"
    assert np.isnan(before).all() and np.isnan(after).all(), desc
    print(f"{shape}: {desc}")


def _tn_table():
    import json
    import os
    path = os.path.join(os.path.dirname(hg.__file__), "csrc", "dispatch_tuning_log_tn.jsonl")
    return {tuple(r["shape"]): r["spec"] for r in (json.loads(line) for line in open(path) if line.strip())}


@pytest.mark.parametrize("shape", [*wl.C2_SHAPES, *wl.C3_SHAPES, wl.C5_SHAPES[0], *wl.c4_shapes()[::5]], ids=lambda s: "x".join(map(str, s)))
def test_column_major_b_with_the_plans_tuned_for_that_layout(shape):
    """B stored N x K (the TN layout of Section 2.2.2) at the benchmark's sizes: the plan is the row of the table
    tuned in that layout, the result is checked at sampled positions against the oracle (real inputs, tolerance)
    and, on the exact-integer family of the shape, bit for bit."""
    cfg = "C2" if shape in wl.C2_SHAPES else "C3" if shape in wl.C3_SHAPES else "C5" if shape in wl.C5_SHAPES else "C4"
    a, b = {"C2": wl.c2_inputs, "C3": wl.c3_inputs, "C4": wl.c4_inputs, "C5": wl.c5_inputs}[cfg](shape)
    c, before, after, desc = run_hgemm(a, np.ascontiguousarray(b.T), b_col_major=True, guard=1)
    want = _tn_table().get(tuple(shape))
    assert want is not None and desc.replace(",pad=1", "") == want, (shape, desc, want)
    _check_sampled(a, b, c, 1500, f"TN {cfg} {shape} {desc}")
    assert np.isnan(before).all() and np.isnan(after).all()
    del a, b, c
    name, ai, bi = wl.exact_family_for(shape, seed=17)
    ci, _, _, _ = run_hgemm(ai, np.ascontiguousarray(bi.T), b_col_major=True)
    ii, jj = wl.sample_positions(shape, 1500, seed=5)
    ref = orc.hgemm_at(ai, bi, ii, jj)
    sel = np.abs(ref.astype(np.float64)) <= 2048
    assert sel.mean() > 0.5, name
    assert np.array_equal(ci[ii, jj][sel].astype(np.float64), ref[sel].astype(np.float64)), f"TN {shape} {name} {desc}"


@pytest.mark.parametrize("b_col_major", [False, True], ids=["NN", "TN"])
@pytest.mark.parametrize("shape", [(3000, 5120, 5120), (8192, 2048, 7168), (3000, 6144, 4096), (11088, 11880, 432), (1000, 8192, 8192)],
                         ids=lambda s: "x".join(map(str, s)))
def test_large_shapes_off_the_table_take_a_tuned_neighbours_kernel_or_the_models(shape, b_col_major):
    """Large problems that the dispatch table does not hold: the planner takes the kernel tuned for the nearest
    shape of the table unless that kernel's tiles fill the last round of workgroups much worse than the cost
    model's pick (3000 x 6144 x 4096 is such a case), and whichever it takes must agree with the oracle at
    sampled positions, bit for bit on the exact-integer family of the shape."""
    name, a, b = wl.exact_family_for(shape, seed=31)
    bb = np.ascontiguousarray(b.T) if b_col_major else b
    c, before, after, desc = run_hgemm(a, bb, b_col_major=b_col_major, guard=1)
    assert desc.startswith("mfma,"), desc
    ii, jj = wl.sample_positions(shape, 3000, seed=6)
    ref = orc.hgemm_at(a, b, ii, jj)
    sel = np.abs(ref.astype(np.float64)) <= 2048
    assert sel.mean() > 0.5, name
    assert np.array_equal(c[ii, jj][sel].astype(np.float64), ref[sel].astype(np.float64)), f"{shape} {name} {desc}"
    assert np.isnan(before).all() and np.isnan(after).all(), desc
    print(f"{shape} {'TN' if b_col_major else 'NN'}: {desc}")


@pytest.mark.parametrize("nk", [*wl.C3_LARGE_NK, *wl.C3_OTHER_NK], ids=lambda nk: f"N{nk[0]}xK{nk[1]}")
def test_llm_projections_of_other_models(nk):
    """The C3 kind of shape for other model widths (beyond the five configurations; C3's input recipe): widths
    8192 and 28672, whose rows for M = 1 and 16 the streaming kernel family holds in the dispatch table, and
    5120 / 13824 / 15360, 6144 x 4096, 10240 x 8192.  One B per (N, K), the first M rows of one A; sampled
    positions against the oracle, and the exact-integer family bit for bit."""
    N, K = nk
    large = nk in wl.C3_LARGE_NK
    ms = wl.C3_LARGE_M if large else wl.C3_M
    top = max(ms)
    a_top, b = wl.c3_inputs((top, N, K))
    _, ai_top, bi = wl.exact_family_for((top, N, K), seed=41)
    for M in ms:
        a = np.ascontiguousarray(a_top[:M])
        c, before, after, desc = run_hgemm(a, b, guard=1)
        if large and M <= 16:
            assert desc.startswith("skinny"), desc
        _check_sampled(a, b, c, 2000, f"{(M, N, K)} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all(), desc
        ai = np.ascontiguousarray(ai_top[:M])
        ci, _, _, _ = run_hgemm(ai, bi)
        ii, jj = wl.sample_positions((M, N, K), 2000, seed=8)
        ref = orc.hgemm_at(ai, bi, ii, jj)
        sel = np.abs(ref.astype(np.float64)) <= 2048
        assert sel.mean() > 0.5
        assert np.array_equal(ci[ii, jj][sel].astype(np.float64), ref[sel].astype(np.float64)), f"{(M, N, K)} {desc}"
        print(f"{(M, N, K)}: {desc}")
    # column-major B: the rows of the table tuned in that layout
    bit = np.ascontiguousarray(bi.T)
    for M in (1, 16):
        ai = np.ascontiguousarray(ai_top[:M])
        ci, _, _, desc = run_hgemm(ai, bit, b_col_major=True)
        assert hg.plan_choice(M, N, K, hg.Layouts.make(b_col_major=True)) == "table: " + desc
        ii, jj = wl.sample_positions((M, N, K), 2000, seed=9)
        ref = orc.hgemm_at(ai, bi, ii, jj)
        sel = np.abs(ref.astype(np.float64)) <= 2048
        assert np.array_equal(ci[ii, jj][sel].astype(np.float64), ref[sel].astype(np.float64)), f"TN {(M, N, K)} {desc}"
