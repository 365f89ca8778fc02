"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2512_02551_amd as hg  # noqa: E402
import workloads as wl  # noqa: E402
from oracle import hgemm_oracle as orc  # noqa: E402

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import assert_bit_exact, assert_close, run_hgemm, to_dev, to_host  # noqa: E402


def all_mfma_specs(sk=1, gm=8):
    out = []
    for line in hg.spec_help().splitlines():
        if "compiled" in line:
            for tup in line.split(":")[1].split():
                bm, bn, bk, wm, wn, st, pf = (int(x) for x in tup.strip("()").split(","))
                out.append(f"mfma,bm={bm},bn={bn},bk={bk},wm={wm},wn={wn},st={st},pf={pf},sk={sk},gm={gm}")
    assert out
    return out


# ---- configuration C1: 256^3 uniform[-1,1], seed 0 -------------------------------------------

def test_c1_256_cubed_default_plan():
    a, b = wl.c1_inputs()
    ref = orc.hgemm(a, b)
    c, _, _, desc = run_hgemm(a, b)
    print("C1 plan:", desc)
    assert_close(c, ref, "C1 " + desc)


# ---- every compiled specialisation, ragged shape, exact integers ------------------------------

@pytest.mark.parametrize("shape", [(300, 264, 200), (33, 520, 328), (257, 72, 64)])
def test_every_spec_bit_exact_on_small_integers_ragged(shape):
    name, a, b = wl.exact_family_for(shape, seed=1)
    ref = orc.hgemm(a, b)
    for spec in all_mfma_specs():
        c, before, after, desc = run_hgemm(a, b, spec=spec, guard=4)
        assert_bit_exact(c, ref, f"{shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all(), f"{desc}: wrote outside C"


@pytest.mark.parametrize("shape", [(300, 264, 200), (33, 520, 328)])
def test_every_spec_tn_layout_bit_exact(shape):
    """B stored column-major (N x K), the paper's TN layout (Section 2.2.2)."""
    name, a, b = wl.exact_family_for(shape, seed=5)
    ref = orc.hgemm(a, b)
    bt = np.ascontiguousarray(b.T)
    assert np.array_equal(orc.hgemm(a, bt, b_col_major=True).view(np.uint16), ref.view(np.uint16))
    for spec in all_mfma_specs() + all_mfma_specs(sk=2):
        c, before, after, desc = run_hgemm(a, bt, spec=spec, b_col_major=True, guard=2)
        assert_bit_exact(c, ref, f"TN {shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all()


def test_tn_default_plan_and_real_inputs():
    shape = (260, 392, 712)
    rng = np.random.default_rng(31)
    a = wl.uniform_pm1(rng, shape[0], shape[2])
    b = wl.uniform_pm1(rng, shape[2], shape[1])
    ref = orc.hgemm(a, b)
    c, _, _, desc = run_hgemm(a, np.ascontiguousarray(b.T), b_col_major=True)
    assert desc.startswith("mfma")
    assert_close(c, ref, "TN " + desc)


@pytest.mark.parametrize("shape", [(300, 264, 200), (1024, 520, 328)])
def test_pretransposed_b_option_bit_exact(shape):
    name, a, b = wl.exact_family_for(shape, seed=6)
    ref = orc.hgemm(a, b)
    for spec in ("mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=2,sk=1,gm=8,tb=1", "mfma,bm=256,bn=256,bk=64,wm=2,wn=4,st=2,sk=2,gm=8,tb=1"):
        c, before, after, desc = run_hgemm(a, b, spec=spec, guard=2)
        assert "tb=1" in desc
        assert_bit_exact(c, ref, f"{shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all()


@pytest.mark.parametrize("shape", [(1312, 1088, 512), (300, 264, 1000), (2100, 2050 // 8 * 8, 328)])
def test_stream_k_bit_exact(shape):
    """Stream-K: tiles that do not fill whole waves of 256 workgroups are shared by K-tile iterations."""
    name, a, b = wl.exact_family_for(shape, seed=7)
    ref = orc.hgemm(a, b)
    ran = 0
    for spec in all_mfma_specs():
        spec = spec + ",sm=1"
        c, before, after, desc = run_hgemm(a, b, spec=spec, guard=2)
        ran += "sm=1" in desc          # the plan drops sm when the tile count is a whole number of waves
        assert_bit_exact(c, ref, f"{shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all()
    assert ran > 0
    bt = np.ascontiguousarray(b.T)
    c, _, _, desc = run_hgemm(a, bt, spec="mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,sk=1,gm=8,sm=1", b_col_major=True)
    assert_bit_exact(c, ref, f"TN {shape} {desc}")


def test_stream_k_real_inputs_and_determinism():
    shape = (1100, 1288, 2048)
    rng = np.random.default_rng(41)
    a = wl.uniform_pm1(rng, shape[0], shape[2])
    b = wl.uniform_pm1(rng, shape[2], shape[1])
    ref = orc.hgemm(a, b)
    for spec in ("mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=2,sk=1,gm=8,sm=1", "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,sk=1,gm=0,sm=1",
                 "mfma,bm=256,bn=256,bk=64,wm=2,wn=4,st=2,sk=1,gm=8,sm=1"):
        c1, _, _, desc = run_hgemm(a, b, spec=spec)
        c2, _, _, _ = run_hgemm(a, b, spec=spec)
        assert "sm=1" in desc
        assert_close(c1, ref, desc)
        assert np.array_equal(c1.view(np.uint16), c2.view(np.uint16)), desc


@pytest.mark.parametrize("sk", [2, 3, 5])
def test_split_k_bit_exact_and_ordered(sk):
    shape = (96, 136, 1000)
    name, a, b = wl.exact_family_for(shape, seed=2)
    ref = orc.hgemm(a, b)
    for spec in all_mfma_specs(sk=sk):
        c, before, after, desc = run_hgemm(a, b, spec=spec, guard=2)
        assert_bit_exact(c, ref, f"{shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all()


@pytest.mark.parametrize("sk", [2, 3, 5])
def test_fused_split_k_bit_exact_every_spec(sk):
    """Split-K with the reduction inside the kernel (fr=1): the last-arriving workgroup of a tile sums the
    planes in split order, so integer inputs are exact and real inputs give the bits of the two-launch form."""
    shape = (96, 136, 1000)
    name, a, b = wl.exact_family_for(shape, seed=2)
    ref = orc.hgemm(a, b)
    rng = np.random.default_rng(77)
    ar = wl.uniform_pm1(rng, shape[0], shape[2])
    br = wl.uniform_pm1(rng, shape[2], shape[1])
    for spec in all_mfma_specs(sk=sk):
        c, before, after, desc = run_hgemm(a, b, spec=spec + ",fr=1", guard=2)
        assert "fr=1" in desc
        assert_bit_exact(c, ref, f"{shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all()
        two, _, _, _ = run_hgemm(ar, br, spec=spec)
        one, _, _, _ = run_hgemm(ar, br, spec=spec + ",fr=1")
        assert np.array_equal(one.view(np.uint16), two.view(np.uint16)), desc


def test_fused_split_k_many_tiles_repeated_launches_and_tn():
    """Many tiles and splits, the same plan launched again and again (the arrival counters must come back to
    zero by themselves), ragged edges, and the column-major B layout."""
    shape = (200, 2056, 4104)
    name, a, b = wl.exact_family_for(shape, seed=9)
    ii, jj = wl.sample_positions(shape, 4000, seed=7, tile=32)
    ref = orc.hgemm_at(a, b, ii, jj).astype(np.float64)
    sel = np.abs(ref) <= 2048
    assert sel.mean() > 0.5
    da, db = to_dev(a), to_dev(b)
    dbt = to_dev(np.ascontiguousarray(b.T))
    sh = torch.cuda.current_stream().cuda_stream
    for spec, tn in (("mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=16,gm=8,fr=1", False),
                     ("mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=1,sk=7,gm=8,fr=1", False),
                     ("mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=3,pf=3,sk=4,gm=8,fr=1", True)):
        with hg.Plan(*shape, hg.Layouts.make(b_col_major=tn), spec) as p:
            first = None
            for rep in range(6):
                c = torch.full((shape[0], shape[1]), float("nan"), dtype=torch.float16, device="cuda")
                p.run(da.data_ptr(), (dbt if tn else db).data_ptr(), c.data_ptr(), sh)
                torch.cuda.synchronize()
                got = to_host(c)
                assert np.array_equal(got[ii, jj].astype(np.float64)[sel], ref[sel]), f"{spec} launch {rep}"
                if first is None:
                    first = got
                assert np.array_equal(got.view(np.uint16), first.view(np.uint16)), f"{spec} launch {rep} differs from launch 0"


def test_persistent_mode_every_capable_spec_bit_exact():
    """Persistent workgroups (ps=1): one per compute unit walks tiles wg, wg + grid, ...; the copies of the next tile
    start under the last K-tiles of the current one and the epilogue stages in the one vacated buffer.  Ragged M and
    N for every tile size, more tiles than compute units (up to 35 tiles per workgroup), a tile count that is not a
    multiple of the grid, both B layouts, several tile orders."""
    shape = (4360, 4104, 520)
    name, a, b = wl.exact_family_for(shape, seed=31)
    ref = orc.hgemm(a, b)
    bt = np.ascontiguousarray(b.T)
    ran = 0
    for spec in all_mfma_specs():
        try:
            c, before, after, desc = run_hgemm(a, b, spec=spec + ",ps=1", guard=2)
        except hg.HgemmError:
            continue                                   # this configuration cannot stage its epilogue in one buffer
        if "ps=1" not in desc:
            continue                                   # too few tiles or K-tiles for this configuration
        ran += 1
        assert_bit_exact(c, ref, f"{shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all(), desc
        if ran % 4 == 0:
            c, _, _, desc = run_hgemm(a, bt, spec=spec.replace("gm=8", "gm=3") + ",ps=1", b_col_major=True)
            assert_bit_exact(c, ref, f"TN {shape} {name} {desc}")
    assert ran >= 30, ran
    # real inputs, run twice: same bits; and the same bits as the non-persistent kernel (same summation order)
    rng = np.random.default_rng(32)
    ar = wl.uniform_pm1(rng, shape[0], shape[2])
    br = wl.uniform_pm1(rng, shape[2], shape[1])
    for spec in ("mfma,bm=256,bn=256,bk=64,wm=2,wn=4,st=2,pf=1,sk=1,gm=8", "mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=4,pf=3,sk=1,gm=0"):
        plain, _, _, _ = run_hgemm(ar, br, spec=spec)
        p1, _, _, desc = run_hgemm(ar, br, spec=spec + ",ps=1")
        p2, _, _, _ = run_hgemm(ar, br, spec=spec + ",ps=1")
        assert "ps=1" in desc
        assert np.array_equal(p1.view(np.uint16), p2.view(np.uint16)) and np.array_equal(p1.view(np.uint16), plain.view(np.uint16)), desc


def _listed_specs(gm=8):
    """(spec, deep) for the configurations spec_help lists on lines of their own: the deep-staged ones (prefetch distance
    longer than a K-tile: one full-K tile per workgroup only) and those built on the 16 x 16 x 32 matrix-core instruction
    (mi=16, a k-step is 32 k)."""
    out = []
    for line in hg.spec_help().splitlines():
        head = line.strip()
        if head.startswith("deep (bm") or head.startswith("mi16 (bm"):
            mi16 = head.startswith("mi16")
            for tup in line.split(":")[1].split():
                bm, bn, bk, wm, wn, st, pf = (int(x) for x in tup.strip("()").split(","))
                spec = f"mfma,bm={bm},bn={bn},bk={bk},wm={wm},wn={wn},st={st},pf={pf},sk=1,gm={gm}" + (",mi=16" if mi16 else "")
                ks = bk // (32 if mi16 else 16)                 # k-steps per K-tile
                out.append((spec, pf > ks or ks == 1))
    assert any("mi=16" in s for s, _ in out) and any("mi=16" not in s for s, _ in out)
    return out


def deep_specs(gm=8):
    return [s for s, deep in _listed_specs(gm) if deep]


def mi16_specs(gm=8):
    return [s for s, deep in _listed_specs(gm) if not deep and "mi=16" in s]


@pytest.mark.parametrize("shape", [(300, 264, 200), (257, 520, 328), (512, 512, 40), (260, 304, 8), (520, 264, 2056), (1030, 1544, 96)])
def test_deep_staged_specs_bit_exact_on_ragged_shapes_both_layouts(shape):
    """Deep-staged configurations (prefetch distance longer than a K-tile): fragment reads run up to two K-tiles ahead
    of the matrix cores and K-tiles past the end are copied as zeros.  K gives an odd and an even number of K-tiles,
    fewer K-tiles than stages (40, 8), a last K-tile of 8 (200, 328, 40, 8, 2056); M and N are ragged; several tiles per
    compute unit in the last shape."""
    name, a, b = wl.exact_family_for(shape, seed=71)
    ref = orc.hgemm(a, b)
    bt = np.ascontiguousarray(b.T)
    for spec in deep_specs() + deep_specs(gm=0):
        c, before, after, desc = run_hgemm(a, b, spec=spec, guard=2)
        assert_bit_exact(c, ref, f"{shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all(), desc
        c, _, _, desc = run_hgemm(a, bt, spec=spec, b_col_major=True)
        assert_bit_exact(c, ref, f"TN {shape} {name} {desc}")


def test_deep_staged_specs_real_inputs_repeatable_and_refusals():
    shape = (520, 776, 4104)
    rng = np.random.default_rng(72)
    a = wl.uniform_pm1(rng, shape[0], shape[2])
    b = wl.uniform_pm1(rng, shape[2], shape[1])
    ref = orc.hgemm(a, b)
    for spec in deep_specs():
        c1, _, _, desc = run_hgemm(a, b, spec=spec)
        c2, _, _, _ = run_hgemm(a, b, spec=spec)
        assert_close(c1, ref, desc)
        assert np.array_equal(c1.view(np.uint16), c2.view(np.uint16)), desc
        for bad in (spec.replace("sk=1", "sk=2"), spec + ",sm=1", spec + ",ps=1", spec + ",ac=16", spec.replace("sk=1", "sk=2") + ",fr=1"):
            with pytest.raises(hg.HgemmError):
                hg.Plan(*shape, None, bad)


@pytest.mark.parametrize("shape", [(300, 264, 200), (257, 520, 328), (520, 776, 2056), (1030, 1544, 96)])
def test_16_wide_matrix_core_blocks_bit_exact_in_every_mode_both_layouts(shape):
    """v_mfma_f32_16x16x32_f16 configurations (mi=16): other fragment and accumulator layouts, the same result.  One
    tile per workgroup, split-K (two launches and fused), stream-K and persistent mode, ragged M, N and K, both
    layouts of B; the 16-bit accumulator is refused (its rounding step is the 16-product step of the 32-wide blocks)."""
    name, a, b = wl.exact_family_for(shape, seed=73)
    ref = orc.hgemm(a, b)
    bt = np.ascontiguousarray(b.T)
    specs = mi16_specs()
    assert specs
    for spec in specs:
        for variant in (spec, spec.replace("sk=1", "sk=3"), spec.replace("sk=1", "sk=2") + ",fr=1", spec + ",sm=1", spec + ",ps=1"):
            c, before, after, desc = run_hgemm(a, b, spec=variant, guard=2)
            assert_bit_exact(c, ref, f"{shape} {name} {desc}")
            assert np.isnan(before).all() and np.isnan(after).all(), desc
            c, _, _, desc = run_hgemm(a, bt, spec=variant, b_col_major=True)
            assert_bit_exact(c, ref, f"TN {shape} {name} {desc}")
        with pytest.raises(hg.HgemmError):
            hg.Plan(*shape, None, spec + ",ac=16")


def test_server_mode_idle_gaps_between_calls():
    """Server mode (Section 2.4.2): the device idles for a random 0-2 ms before every call, caches and clocks cool
    down in between.  Every call of a plan, whatever its kind (single kernel, two-launch split-K, fused split-K
    with its self-resetting counters, stream-K, persistent, skinny), must still give the oracle's result."""
    import random
    import time

    rnd = random.Random(7)
    shape = (200, 2056, 1288)
    name, a, b = wl.exact_family_for(shape, seed=51)
    ref = orc.hgemm(a, b)
    da, db = to_dev(a), to_dev(b)
    sh = torch.cuda.current_stream().cuda_stream
    specs = [None, "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=3,sk=3,gm=8", "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=3,sk=5,gm=8,fr=1",
             "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=1,sk=1,gm=8,sm=1", "mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=1,gm=8,ps=1"]
    for spec in specs:
        with hg.Plan(*shape, None, spec) as p:
            for call in range(5):
                torch.cuda.synchronize()
                time.sleep(rnd.uniform(0.0, 2e-3))
                c = torch.full((shape[0], shape[1]), float("nan"), dtype=torch.float16, device="cuda")
                p.run(da.data_ptr(), db.data_ptr(), c.data_ptr(), sh)
                torch.cuda.synchronize()
                assert_bit_exact(to_host(c), ref, f"{p.describe()} call {call}")
    shape = (16, 2056, 1288)
    name, a, b = wl.exact_family_for(shape, seed=52)
    ref = orc.hgemm(a, b)
    da, db = to_dev(a), to_dev(b)
    for spec in ("skinny,sk=4", "skinny,sk=4,fr=1"):
        with hg.Plan(*shape, None, spec) as p:
            for call in range(5):
                torch.cuda.synchronize()
                time.sleep(rnd.uniform(0.0, 2e-3))
                c = torch.full((shape[0], shape[1]), float("nan"), dtype=torch.float16, device="cuda")
                p.run(da.data_ptr(), db.data_ptr(), c.data_ptr(), sh)
                torch.cuda.synchronize()
                assert_bit_exact(to_host(c), ref, f"{p.describe()} call {call}")


def test_run_many_equals_a_loop_of_runs_and_rotates_operand_sets():
    """hgemm_run_many (Section 2.4.2's offline mode, the loop inside the library): call i works on operand set
    (first + i) % sets; every set's result must be the oracle's, for single-kernel, two-launch and fused plans,
    and sets that no call reaches stay untouched."""
    shape = (72, 520, 1096)
    sets = []
    for seed in (61, 62, 63, 64):
        name, a, b = wl.exact_family_for(shape, seed=seed)
        sets.append((to_dev(a), to_dev(b), orc.hgemm(a, b)))
    sh = torch.cuda.current_stream().cuda_stream
    for spec in (None, "mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=4,gm=8", "mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=4,gm=8,fr=1"):
        with hg.Plan(*shape, None, spec) as p:
            for count, first in ((4, 0), (9, 2), (2, 3), (0, 1)):
                cs = [torch.full((shape[0], shape[1]), float("nan"), dtype=torch.float16, device="cuda") for _ in sets]
                p.run_many(count, [(a.data_ptr(), b.data_ptr(), c.data_ptr()) for (a, b, _), c in zip(sets, cs)], sh, first)
                torch.cuda.synchronize()
                reached = {(first + i) % len(sets) for i in range(count)}
                for j, ((_, _, ref), c) in enumerate(zip(sets, cs)):
                    if j in reached:
                        assert_bit_exact(to_host(c), ref, f"{p.describe()} count {count} first {first} set {j}")
                    else:
                        assert bool(torch.isnan(c).all()), f"set {j} was written although no call reaches it"
            with pytest.raises(hg.HgemmError):
                p.run_many(1, [(sets[0][0].data_ptr(), sets[0][1].data_ptr(), 0)], sh, 1)      # first >= sets


def skinny_specs(M, N, K):
    out = [c for c in hg.candidates(M, N, K) if c.startswith("skinny")]
    assert out
    return out


@pytest.mark.parametrize("shape", [(1, 264, 200), (16, 520, 1000), (7, 72, 4104), (33, 136, 328), (16, 4096, 32), (5, 8, 8), (64, 200, 776),
                                   (48, 1032, 2056), (17, 128, 64)])
def test_skinny_family_every_spec_bit_exact(shape):
    """The memory-bound family (128-column strips x K slabs in steps of 16 rows per wave, workgroups of 4, 8 or 16
    waves, blocks of B transposed in registers for 16x16x16 matrix-core instructions, the waves' sums added in
    wave order; slabs summed in order by the reduction launch or by the last-arriving workgroup): ragged N, K
    not a multiple of the step or of the slab count, one, two and four 16-row blocks of A, K shorter than a
    step."""
    name, a, b = wl.exact_family_for(shape, seed=12)
    ref = orc.hgemm(a, b)
    rng = np.random.default_rng([shape[0], shape[1], shape[2], 3])
    ar = wl.uniform_pm1(rng, shape[0], shape[2])
    br = wl.uniform_pm1(rng, shape[2], shape[1])
    refr = orc.hgemm(ar, br)
    specs = skinny_specs(*shape)
    assert any("wv=8" in x for x in specs) and any("wv=" not in x for x in specs)
    # 16 waves leave a lane the registers for two 16-row blocks of A
    for spec in specs + ["skinny,sk=3", "skinny,sk=5,fr=1", "skinny,sk=3,wv=8", "skinny,sk=2,fr=1,wv=16" if shape[0] <= 32 else "skinny,sk=2,fr=1,wv=8"]:
        c, before, after, desc = run_hgemm(a, b, spec=spec, guard=3)
        assert desc.startswith("skinny")
        assert_bit_exact(c, ref, f"{shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all(), f"{desc}: wrote outside C"
        c, _, _, _ = run_hgemm(ar, br, spec=spec)
        assert_close(c, refr, f"{shape} real {desc}")
        again, _, _, _ = run_hgemm(ar, br, spec=spec)
        assert np.array_equal(c.view(np.uint16), again.view(np.uint16)), f"{desc}: two runs differ"
    # the fused reduction gives the bits of the two-launch reduction
    two, _, _, _ = run_hgemm(ar, br, spec="skinny,sk=4")
    one, _, _, _ = run_hgemm(ar, br, spec="skinny,sk=4,fr=1")
    assert np.array_equal(one.view(np.uint16), two.view(np.uint16))
    two, _, _, _ = run_hgemm(ar, br, spec="skinny,sk=2,wv=8")
    one, _, _, _ = run_hgemm(ar, br, spec="skinny,sk=2,fr=1,wv=8")
    assert np.array_equal(one.view(np.uint16), two.view(np.uint16))
    # column-major B: 16 columns of C per workgroup, the waves split K, 16-byte loads are the matrix-core operands
    tn = hg.Layouts.make(b_col_major=True)
    bt, brt = np.ascontiguousarray(b.T), np.ascontiguousarray(br.T)
    tn_specs = [c for c in hg.candidates(*shape, tn) if c.startswith("skinny")]
    assert tn_specs and any("wv=8" in x for x in tn_specs)
    # wider workgroups (32 or 64 rows of B) are candidates only for wide N: named here
    for spec in tn_specs + ["skinny,sk=3", "skinny,sk=2,fr=1,wv=8", "skinny,sk=1,nr=32", "skinny,sk=3,nr=64", "skinny,sk=2,fr=1,wv=8,nr=32"]:
        c, before, after, desc = run_hgemm(a, bt, spec=spec, b_col_major=True, guard=3)
        assert desc.startswith("skinny")
        assert_bit_exact(c, ref, f"TN {shape} {name} {desc}")
        assert np.isnan(before).all() and np.isnan(after).all(), f"TN {desc}: wrote outside C"
        c, _, _, _ = run_hgemm(ar, brt, spec=spec, b_col_major=True)
        assert_close(c, refr, f"TN {shape} real {desc}")
        again, _, _, _ = run_hgemm(ar, brt, spec=spec, b_col_major=True)
        assert np.array_equal(c.view(np.uint16), again.view(np.uint16)), f"TN {desc}: two runs differ"
    two, _, _, _ = run_hgemm(ar, brt, spec="skinny,sk=2,wv=8", b_col_major=True)
    one, _, _, _ = run_hgemm(ar, brt, spec="skinny,sk=2,fr=1,wv=8", b_col_major=True)
    assert np.array_equal(one.view(np.uint16), two.view(np.uint16))


def test_skinny_family_repeated_launches_padded_leading_dimensions_and_refusals():
    M, N, K = 12, 328, 2056
    name, a, b = wl.exact_family_for((M, N, K), seed=14)
    ref = orc.hgemm(a, b)
    lda, ldb, ldc = K + 24, N + 40, N + 8
    A = torch.full((M, lda), float("nan"), dtype=torch.float16, device="cuda")
    B = torch.full((K, ldb), float("nan"), dtype=torch.float16, device="cuda")
    C = torch.full((M, ldc), float("nan"), dtype=torch.float16, device="cuda")
    A[:, :K] = to_dev(a)
    B[:, :N] = to_dev(b)
    for spec in ("skinny,sk=1", "skinny,sk=4", "skinny,sk=8,fr=1", "skinny,sk=1,wv=16", "skinny,sk=4,wv=8", "skinny,sk=8,fr=1,wv=8"):
        with hg.Plan(M, N, K, hg.Layouts.make(lda=lda, ldb=ldb, ldc=ldc), spec) as p:
            for rep in range(4):            # the arrival counters of the fused form come back to zero by themselves
                C.fill_(float("nan"))
                p.run(A.data_ptr(), B.data_ptr(), C.data_ptr(), torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
                out = to_host(C)
                assert_bit_exact(out[:, :N], ref, f"{spec} launch {rep}")
                assert np.isnan(out[:, N:]).all(), spec
    # unaligned shapes and tall A are not this family's
    with pytest.raises(hg.HgemmError):
        hg.Plan(8, 60, 64, None, "skinny,sk=1")
    with pytest.raises(hg.HgemmError):
        hg.Plan(64, 64, 64, hg.Layouts.make(b_col_major=True), "skinny,sk=1,wv=8,nr=64")      # sums beyond 64 KiB of LDS
    with pytest.raises(hg.HgemmError):
        hg.Plan(16, 64, 64, None, "skinny,sk=1,nr=32")                                       # row-major B has 128-column strips
    with pytest.raises(hg.HgemmError):
        hg.Plan(65, 64, 64, None, "skinny,sk=1")
    with pytest.raises(hg.HgemmError):
        hg.Plan(64, 64, 64, None, "skinny,sk=1,wv=16")          # 16 waves: two 16-row blocks of A at most
    with pytest.raises(hg.HgemmError):
        hg.Plan(16, 64, 64, None, "skinny,sk=1,wv=5")
    with pytest.raises(hg.HgemmError):
        hg.Plan(64, 64, 64, None, "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=3,sk=1,gm=8,wv=8")


@pytest.mark.parametrize("spec", ["skinny,sk=1", "skinny,sk=2", "skinny,sk=3,fr=1", "skinny,sk=1,wv=8", "skinny,sk=1,wv=16"])
def test_skinny_family_non_finite_and_subnormal_values(spec):
    """NaN and infinities in A or B reach exactly the elements of C the definition gives them (a kernel that
    multiplied a value of B with a zero that is not A's would spread them to neighbouring columns), an
    infinity times a zero of the other operand is NaN, and subnormal inputs and results are kept."""
    M, N, K = 13, 264, 200
    a, b = wl.small_int_inputs((M, N, K), seed=9)
    a = a.copy()
    b = b.copy()
    a[3, 5] = np.nan
    a[10, 64] = np.inf
    b[64, 7] = 0              # inf * 0 = NaN at C[10, 7]
    b[17, 130] = np.inf       # a whole column of +-inf or, where A[m][17] == 0, NaN: column 130 only
    b[199, 263] = np.nan
    ref = orc.hgemm(a, b)
    for tn in (False, True):
        c, _, _, desc = run_hgemm(a, np.ascontiguousarray(b.T) if tn else b, spec=spec, b_col_major=tn)
        assert np.array_equal(np.isnan(c), np.isnan(ref)), desc
        fin = ~np.isnan(ref)
        assert np.array_equal(c[fin].astype(np.float64), ref[fin].astype(np.float64)), desc
    clean = [m for m in range(M) if m not in (3, 10)]          # rows of A without a non-finite value
    assert np.isfinite(ref[clean, 129]).all() and np.isfinite(ref[clean, 131]).all() and not np.isfinite(ref[:, 130]).any()
    rng = np.random.default_rng(78)
    a2 = (rng.integers(-3, 4, size=(M, K)).astype(np.float64) * 2.0 ** -24).astype(np.float16)
    b2 = wl.integers(rng, K, N, -2, 2)
    ref2 = orc.hgemm(a2, b2)
    assert (np.abs(ref2.astype(np.float64)) < 2.0 ** -14).all() and np.count_nonzero(ref2) > M * N // 2
    c2, _, _, desc = run_hgemm(a2, b2, spec=spec)
    assert_bit_exact(c2, ref2, "subnormal A: " + desc)


def test_every_spec_real_inputs_within_tolerance():
    shape = (520, 392, 712)
    rng = np.random.default_rng(3)
    a = wl.uniform_pm1(rng, shape[0], shape[2])
    b = wl.uniform_pm1(rng, shape[2], shape[1])
    ref = orc.hgemm(a, b)
    for spec in all_mfma_specs() + all_mfma_specs(sk=3):
        c, _, _, desc = run_hgemm(a, b, spec=spec)
        assert_close(c, ref, desc)


# ---- the paper's binary exact-match test (Section 2.3.2), several seeds ------------------------

@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4])
def test_binary_exact_match_below_2048(seed):
    shape = (128, 192, 4096)
    a, b = wl.binary_inputs(shape, seed=seed)
    ref = orc.hgemm(a, b)
    c, _, _, desc = run_hgemm(a, b)
    r = ref.astype(np.float64)
    sel = r <= 2048
    assert sel.mean() > 0.9 and (r > 0).mean() > 0.9
    assert np.array_equal(c.astype(np.float64)[sel], r[sel]), desc


def test_half_integer_inputs_exact_below_1024():
    shape = (64, 128, 1024)
    rng = np.random.default_rng(5)
    a = wl.bernoulli(rng, shape[0], shape[2], 0.6, 0.5)
    b = wl.bernoulli(rng, shape[2], shape[1], 0.6, 1.0)
    ref = orc.hgemm(a, b)
    c, _, _, desc = run_hgemm(a, b)
    sel = ref.astype(np.float64) < 1024
    assert sel.all()
    assert_bit_exact(c, ref, desc)


# ---- tile order, tails, degenerate shapes -------------------------------------------------------

@pytest.mark.parametrize("gm", [0, 1, 3, 8, 16])
def test_tile_order_variants(gm):
    shape = (40 * 32, 35 * 64, 64)          # 40 x 35 tiles of 32x64... many workgroups, not a multiple of 256
    name, a, b = wl.exact_family_for(shape, seed=gm)
    ref = orc.hgemm(a, b)
    for spec in (f"mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,sk=1,gm={gm}", f"mfma,bm=32,bn=128,bk=64,wm=1,wn=4,st=4,sk=1,gm={gm}"):
        c, _, _, desc = run_hgemm(a, b, spec=spec)
        assert_bit_exact(c, ref, desc)


@pytest.mark.parametrize("shape", [(1, 64, 64), (1, 4096, 512), (16, 128, 4096), (7, 8, 8), (5, 72, 24), (64, 64, 8)])
def test_small_m_and_tiny_shapes_default_plan(shape):
    name, a, b = wl.exact_family_for(shape, seed=3)
    ref = orc.hgemm(a, b)
    c, before, after, desc = run_hgemm(a, b, guard=3)
    if name == "binary":
        sel = ref.astype(np.float64) <= 2048
        assert np.array_equal(c[sel].view(np.uint16), ref[sel].view(np.uint16)), desc
    else:
        assert_bit_exact(c, ref, f"{shape} {desc}")
    assert np.isnan(before).all() and np.isnan(after).all()


def _random_shapes(count, seed):
    """Dimensions log-uniform over 1 .. 4096, two thirds of them rounded to multiples of 8 (the matrix-core path),
    the rest left as drawn (padded copies or the generic kernel); M*N*K bounded so that the oracle stays quick."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        dims = [int(2.0 ** rng.uniform(0.0, 12.0)) for _ in range(3)]
        if rng.random() < 2.0 / 3.0:
            dims[1] = max(8, dims[1] // 8 * 8)
            dims[2] = max(8, dims[2] // 8 * 8)
        if dims[0] * dims[1] * dims[2] <= 3e8:
            out.append(tuple(dims))
    return out


def test_random_shapes_whatever_the_planner_picks_both_layouts():
    """160 seeded random shapes and two large skinny ones through hgemm_plan (dispatch table never hit: cost model,
    nearest tuned shape, streaming family, padded copies, generic kernel), row-major and column-major B: bit-exact on {-2..2} inputs
    wherever |C| <= 2048, nothing written outside C, and every family of plan seen at least once."""
    seen = set()
    # two shapes with a few rows of A against weights of 256 MiB: what the planner gives to the streaming family
    shapes = _random_shapes(160, 2024) + [(8, 16384, 8192), (24, 8192, 16384)]
    for i, shape in enumerate(shapes):
        M, N, K = shape
        rng = np.random.default_rng([i, M, N, K])
        a = wl.integers(rng, M, K, -2, 2)
        b = wl.integers(rng, K, N, -2, 2)
        ref = orc.hgemm(a, b)
        sel = np.abs(ref.astype(np.float64)) <= 2048
        tn = i % 3 == 2
        c, before, after, desc = run_hgemm(a, np.ascontiguousarray(b.T) if tn else b, b_col_major=tn, guard=2)
        assert np.array_equal(c[sel].astype(np.float64), ref[sel].astype(np.float64)), f"{shape} {'TN' if tn else 'NN'} {desc}"
        assert not np.isnan(c).any(), f"{shape} {desc}: part of C not written"
        assert np.isnan(before).all() and np.isnan(after).all(), f"{shape} {desc}: wrote outside C"
        seen.add("pad" if "pad=1" in desc else desc.split(",")[0])
        # the host-only preview of the planner's decision names the plan that was set up
        assert hg.plan_choice(M, N, K, hg.Layouts.make(b_col_major=tn)).split(": ")[-1] == desc, (shape, tn)
    assert {"mfma", "skinny", "generic", "pad"} <= seen, seen


@pytest.mark.parametrize("shape", [(3, 5, 7), (17, 9, 33), (65, 130, 100), (1, 1, 1), (129, 63, 100)])
def test_small_unaligned_shapes_take_generic_kernel(shape):
    M, N, K = shape
    rng = np.random.default_rng(sum(shape))
    a = wl.integers(rng, M, K, -3, 3)
    b = wl.integers(rng, K, N, -3, 3)
    ref = orc.hgemm(a, b)
    c, _, _, desc = run_hgemm(a, b)
    assert desc == "generic"
    assert_bit_exact(c, ref, f"{shape}")
    # TN layout (B stored N x K) gives the same product
    c2, _, _, desc2 = run_hgemm(a, np.ascontiguousarray(b.T), b_col_major=True)
    assert desc2 == "generic"
    assert_bit_exact(c2, ref, f"{shape} TN")


def test_empty_and_k_zero():
    # K = 0: C must become all zeros whatever it held
    a = np.zeros((5, 0), dtype=np.float16)
    b = np.zeros((0, 16), dtype=np.float16)
    c, _, _, _ = run_hgemm(a, b, prefill=7.0)
    assert c.shape == (5, 16) and not c.any()
    # ... also for widths that are not multiples of 8 and for a padded leading dimension, touching nothing else
    for (M, N, ldc) in [(7, 13, 13), (300, 2050, 2056), (33, 4099, 4101), (64, 4096, 4096)]:
        dC = torch.full((M + 2, ldc), 7.0, dtype=torch.float16, device="cuda")
        with hg.Plan(M, N, 0, hg.Layouts.make(ldc=ldc)) as p:
            p.run(None, None, dC[1:].data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        out = to_host(dC)
        assert not out[1:M + 1, :N].any(), (M, N, ldc)
        assert (out[0] == 7).all() and (out[M + 1] == 7).all() and (out[1:M + 1, N:] == 7).all(), (M, N, ldc)
    # M = 0 / N = 0: nothing to do, nothing touched
    with hg.Plan(0, 16, 8) as p:
        assert p.run_status(None, None, None) == 0
    with hg.Plan(4, 0, 8) as p:
        assert p.run_status(None, None, None) == 0


def test_beta_zero_semantics_nan_in_c_never_leaks():
    a, b = wl.small_int_inputs((64, 64, 64), seed=9)
    ref = orc.hgemm(a, b)
    c, _, _, desc = run_hgemm(a, b, prefill=float("nan"))
    assert not np.isnan(c).any()
    assert_bit_exact(c, ref, desc)


def test_run_to_run_determinism_on_real_inputs():
    shape = (384, 512, 2048)
    rng = np.random.default_rng(21)
    a = wl.uniform_pm1(rng, shape[0], shape[2])
    b = wl.uniform_pm1(rng, shape[2], shape[1])
    for spec in (None, "mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=4,sk=4,gm=8"):
        c1, _, _, desc = run_hgemm(a, b, spec=spec)
        c2, _, _, _ = run_hgemm(a, b, spec=spec)
        assert np.array_equal(c1.view(np.uint16), c2.view(np.uint16)), desc


def test_nan_and_inf_propagate_like_the_oracle():
    a, b = wl.small_int_inputs((64, 64, 64), seed=4)
    a = a.copy()
    b = b.copy()
    a[3, 5] = np.nan
    a[10, 0] = np.inf
    b[0, 7] = 0          # inf * 0 = NaN at C[10, 7]
    ref = orc.hgemm(a, b)
    c, _, _, desc = run_hgemm(a, b)
    assert np.array_equal(np.isnan(c), np.isnan(ref)), desc
    fin = ~np.isnan(ref)
    assert np.array_equal(c[fin].astype(np.float64), ref[fin].astype(np.float64))


def test_overflow_rounds_to_infinity():
    K = 64
    a = np.full((32, K), 60.0, dtype=np.float16)
    b = np.full((K, 64), 30.0, dtype=np.float16)       # 64 * 1800 = 115200 > 65504
    ref = orc.hgemm(a, b)
    c, _, _, _ = run_hgemm(a, b)
    assert np.isinf(ref).all() and np.array_equal(c.view(np.uint16), ref.view(np.uint16))


@pytest.mark.parametrize("spec", [None, "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=1,sk=2,gm=8", "generic"])
def test_subnormal_inputs_and_outputs_are_not_flushed(spec):
    """fp16 subnormals are ordinary values of the format (Section 2.1 puts no range limit on A, B, C):
    A holds multiples of 2^-24 below the smallest normal, B small integers, so every C element is an
    exactly representable subnormal (|C| <= 3*2*96 units of 2^-24) and must match bit for bit.  A second
    case reaches subnormal results from normal inputs (2^-14 * 2^-10)."""
    M, N, K = 72, 136, 96
    rng = np.random.default_rng(77)
    a = (rng.integers(-3, 4, size=(M, K)).astype(np.float64) * 2.0 ** -24).astype(np.float16)
    b = wl.integers(rng, K, N, -2, 2)
    ref = orc.hgemm(a, b)
    assert (np.abs(ref.astype(np.float64)) < 2.0 ** -14).all() and np.count_nonzero(ref) > M * N // 2
    c, _, _, desc = run_hgemm(a, b, spec=spec)
    assert_bit_exact(c, ref, "subnormal A: " + desc)
    a2 = np.full((M, K), 2.0 ** -14, dtype=np.float16)
    b2 = np.zeros((K, N), dtype=np.float16)
    b2[np.arange(K), np.arange(K)] = 2.0 ** -10          # C[:, j] = 2^-24 for j < K, else 0
    ref2 = orc.hgemm(a2, b2)
    assert ref2[0, 0] == np.float16(2.0 ** -24) and ref2[0, N - 1] == 0
    c2, _, _, desc = run_hgemm(a2, b2, spec=spec)
    assert_bit_exact(c2, ref2, "subnormal C: " + desc)


def test_leading_dimensions():
    M, N, K = 96, 80, 72
    lda, ldb, ldc = 88, 96, 104
    rng = np.random.default_rng(8)
    A = wl.integers(rng, M, lda, -2, 2)
    B = wl.integers(rng, K, ldb, -2, 2)
    ref = orc.hgemm(np.ascontiguousarray(A[:, :K]), np.ascontiguousarray(B[:, :N]))
    dA, dB = to_dev(A), to_dev(B)
    dC = torch.full((M, ldc), float("nan"), dtype=torch.float16, device="cuda")
    lay = hg.Layouts.make(lda=lda, ldb=ldb, ldc=ldc)
    for spec in (None, "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,sk=2,gm=8", "generic"):
        dC.fill_(float("nan"))
        with hg.Plan(M, N, K, lay, spec) as p:
            p.run(dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            desc = p.describe()
        out = to_host(dC)
        assert_bit_exact(out[:, :N], ref, desc)
        assert np.isnan(out[:, N:]).all(), desc + ": wrote into the padding of C"


@pytest.mark.parametrize("shape", [(65, 130, 257), (300, 263, 201), (129, 1001, 515), (1000, 1001, 1003), (33, 4097, 1025), (2050, 77, 130)],
                         ids=lambda s: "x".join(map(str, s)))
def test_unaligned_large_shapes_run_on_zero_padded_copies(shape):
    """N or K not a multiple of 8, problem large enough: the planner pads N and K to 8 in workspace copies
    (zero padding, Section 5.2) and runs the matrix-core kernel; results are still exact, nothing is written
    outside C, and both B layouts agree."""
    M, N, K = shape
    name, a, b = wl.exact_family_for(shape, seed=13)
    ref = orc.hgemm(a, b)
    c, before, after, desc = run_hgemm(a, b, guard=2)
    assert desc.startswith("mfma") and desc.endswith("pad=1"), desc
    assert_bit_exact(c, ref, f"{shape} {name} {desc}")
    assert np.isnan(before).all() and np.isnan(after).all(), desc
    c2, before, after, desc2 = run_hgemm(a, np.ascontiguousarray(b.T), b_col_major=True, guard=2)
    assert desc2.endswith("pad=1"), desc2
    assert_bit_exact(c2, ref, f"TN {shape} {name} {desc2}")
    assert np.isnan(before).all() and np.isnan(after).all(), desc2
    # real inputs, twice with the same plan: the padded copies are rewritten on every call
    rng = np.random.default_rng(shape)
    ar, br = wl.uniform_pm1(rng, M, K), wl.uniform_pm1(rng, K, N)
    cr, _, _, _ = run_hgemm(ar, br)
    assert_close(cr, orc.hgemm(ar, br), f"{shape} real {desc}")


def test_odd_leading_dimensions_run_on_zero_padded_copies():
    M, N, K = 264, 328, 200                      # aligned sizes, leading dimensions that are not multiples of 8
    lda, ldb, ldc = 203, 331, 335
    rng = np.random.default_rng(18)
    A = wl.integers(rng, M, lda, -2, 2)
    B = wl.integers(rng, K, ldb, -2, 2)
    ref = orc.hgemm(np.ascontiguousarray(A[:, :K]), np.ascontiguousarray(B[:, :N]))
    dA, dB = to_dev(A), to_dev(B)
    dC = torch.full((M, ldc), float("nan"), dtype=torch.float16, device="cuda")
    with hg.Plan(M, N, K, hg.Layouts.make(lda=lda, ldb=ldb, ldc=ldc)) as p:
        desc = p.describe()
        assert desc.endswith("pad=1"), desc
        for _ in range(2):
            dC.fill_(float("nan"))
            p.run(dA.data_ptr(), dB.data_ptr(), dC.data_ptr(), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            out = to_host(dC)
            assert_bit_exact(out[:, :N], ref, desc)
            assert np.isnan(out[:, N:]).all(), desc + ": wrote into the padding of C"
    # an explicit matrix-core spec still refuses memory it cannot address with 16-byte copies
    with pytest.raises(hg.HgemmError) as e:
        hg.Plan(M, N, K, hg.Layouts.make(lda=lda, ldb=ldb, ldc=ldc), "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=1,sk=1,gm=8")
    assert e.value.status == 2


def test_error_paths():
    with pytest.raises(hg.HgemmError) as e:
        hg.Plan(-1, 8, 8)
    assert e.value.status == 1
    with pytest.raises(hg.HgemmError) as e:
        hg.Plan(64, 64, 64, None, "mfma,bm=17,bn=64,bk=64,wm=2,wn=2,st=4")
    assert e.value.status == 2
    with pytest.raises(hg.HgemmError) as e:
        hg.Plan(64, 64, 64, None, "nonsense")
    assert e.value.status == 1
    with pytest.raises(hg.HgemmError) as e:
        hg.Plan(64, 64, 63, None, "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4")     # K not a multiple of 8
    assert e.value.status == 2
    lay = hg.Layouts.make()
    lay.a = 1                                                                  # column-major A is not offered
    with pytest.raises(hg.HgemmError) as e:
        hg.Plan(64, 64, 64, lay)
    assert e.value.status == 2
    with hg.Plan(64, 64, 64) as p:
        assert p.run_status(None, None, None) == 1                             # null pointers with work to do


def test_runs_can_be_captured_in_a_graph_and_replayed():
    """hgemm_run only launches kernels on the stream it is given, so a caller may capture it into a
    graph (launch-bound loops of small GEMMs).  Plain, split-K, stream-K and transposing-copy plans are
    captured together, the graph is replayed several times with eager work in between, and every replay
    must reproduce the eager results bit for bit."""
    shape = (300, 520, 1000)
    name, a, b = wl.exact_family_for(shape, seed=9)
    ref = orc.hgemm(a, b)
    specs = [None, "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=1,sk=3,gm=8", "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=1,sk=1,gm=8,sm=1",
             "mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=2,pf=1,sk=1,gm=8,tb=1"]
    da, db = to_dev(a), to_dev(b)
    plans = [hg.Plan(*shape, None, s) for s in specs]
    outs = [torch.full((shape[0], shape[1]), float("nan"), dtype=torch.float16, device="cuda") for _ in plans]
    try:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            cs = torch.cuda.current_stream().cuda_stream
            for p, o in zip(plans, outs):
                p.run(da.data_ptr(), db.data_ptr(), o.data_ptr(), cs)
        for rep in range(3):
            for o in outs:
                o.fill_(float("nan"))
            # unrelated eager work between replays
            c_eager, _, _, _ = run_hgemm(a, b)
            assert_bit_exact(c_eager, ref, "eager between replays")
            g.replay()
            torch.cuda.synchronize()
            for p, o in zip(plans, outs):
                assert_bit_exact(to_host(o), ref, f"replay {rep} {p.describe()}")
    finally:
        for p in plans:
            p.destroy()
