"""CPU-only checks: the library loads, exports every declared symbol, and its host-side logic
(tile arithmetic, tile order) is right.  No kernel is launched here."""
import os
import re

import pytest

import paper_2512_02551_amd as hg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hg.lib_path()):
        from paper_2512_02551_amd import build
        build.build(force=True)
    return hg.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "hgemm.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(hgemm_[a-z_]+)\s*\(", header))
    assert declared == set(hg.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings(lib):
    for s in range(6):
        assert hg.status_string(s)
    assert "gfx950" in hg.status_string(5)


def test_run_entry_points_refuse_a_null_plan_before_touching_the_gpu(lib):
    import ctypes
    one = (ctypes.c_void_p * 1)(0)
    assert lib.hgemm_run(None, None, None, None, None) == 1
    assert lib.hgemm_run_many(None, 1, 1, 0, one, one, one, None) == 1


def test_padding_arithmetic_matches_the_papers_example(lib):
    # Section 5.2: M = 8192, BM = 160 -> 52 tiles, 8320 rows
    assert hg.tiles(8192, 160) == 52
    assert hg.padded(8192, 160) == 8320
    assert hg.tiles(0, 64) == 0 and hg.tiles(1, 64) == 1 and hg.tiles(64, 64) == 1 and hg.tiles(65, 64) == 2
    assert hg.tiles(5, 0) == -1


@pytest.mark.parametrize("tm,tn", [(1, 1), (3, 5), (32, 32), (16, 16), (40, 35), (7, 300), (300, 7), (64, 43), (1, 1000)])
@pytest.mark.parametrize("group", [0, 1, 3, 8, 16])
def test_tile_order_is_a_bijection(lib, tm, tn, group):
    total = tm * tn
    seen = [hg.tile_of_workgroup(w, tm, tn, group) for w in range(total)]
    assert sorted(seen) == list(range(total))
    assert hg.tile_of_workgroup(total, tm, tn, group) == -1


def test_tile_order_keeps_an_xcd_on_a_compact_block(lib):
    # 32 x 32 tiles, group 8: the 32 workgroups one XCD gets from a run of 256 ids
    # (ids congruent mod 8) must cover 8 tile-rows x 4 tile-columns.
    tm = tn = 32
    for xcd in range(8):
        tiles = [hg.tile_of_workgroup(w, tm, tn, 8) for w in range(xcd, 256, 8)]
        rows = {t // tn for t in tiles}
        cols = {t % tn for t in tiles}
        assert len(rows) == 8 and len(cols) == 4
    # and a whole run of 256 ids covers 8 rows x 32 columns
    tiles = [hg.tile_of_workgroup(w, tm, tn, 8) for w in range(256)]
    assert {t // tn for t in tiles} == set(range(8)) and {t % tn for t in tiles} == set(range(32))


def test_candidates_and_help_are_consistent(lib):
    specs = hg.candidates(4096, 4096, 4096)
    assert specs and all(s.startswith("mfma,") for s in specs)
    assert hg.candidates(3, 5, 7) == ["generic"]
    text = hg.spec_help()
    assert "generic" in text and "mfma" in text
    skinny = hg.candidates(16, 4096, 4096)
    assert any("sk=8" in s or "sk=16" in s for s in skinny)


# ---- randomised host-side properties ----------------------------------------------------------------

from hypothesis import given, settings, strategies as hst  # noqa: E402


@settings(max_examples=60, deadline=None)
@given(tm=hst.integers(1, 70), tn=hst.integers(1, 70), group=hst.sampled_from([0, 1, 2, 3, 4, 8, 16, 64]))
def test_tile_order_is_a_permutation_for_random_grids(tm, tn, group):
    import paper_2512_02551_amd as hg
    seen = sorted(hg.tile_of_workgroup(w, tm, tn, group) for w in range(tm * tn))
    assert seen == list(range(tm * tn))
    assert hg.tile_of_workgroup(tm * tn, tm, tn, group) == -1            # one past the end is refused


@settings(max_examples=200, deadline=None)
@given(dim=hst.integers(0, 1 << 24), tile=hst.sampled_from([8, 32, 64, 128, 160, 256]))
def test_padding_arithmetic_properties(dim, tile):
    import paper_2512_02551_amd as hg
    t, p = hg.tiles(dim, tile), hg.padded(dim, tile)
    assert p == t * tile and p >= dim and p - dim < tile


@settings(max_examples=40, deadline=None)
@given(M=hst.integers(1, 20000), N8=hst.integers(1, 2500), K8=hst.integers(1, 2500))
def test_every_candidate_has_a_finite_positive_prediction(M, N8, K8):
    """The planner takes the minimum of the cost model over these candidates, so the model has to be
    defined (finite, positive) on every one of them, for any aligned shape."""
    import math

    import paper_2512_02551_amd as hg
    N, K = 8 * N8, 8 * K8
    cands = [s for s in hg.candidates(M, N, K) if "sm=1" not in s and "tb=1" not in s and "ps=1" not in s]
    assert cands and all(s.startswith(("mfma,", "skinny,")) for s in cands)
    for s in cands[::3]:
        us = hg.predict_us(M, N, K, s)
        assert math.isfinite(us) and us > 1.0, (M, N, K, s, us)


def test_plan_choice_names_the_source_of_every_kind_of_plan():
    """hgemm_plan_choice is the planner's decision without a device: dispatch table, nearest tuned shape for large
    problems off the table (unless its tiles fill the last round of workgroups worse than the model's pick),
    cost model, streaming family for a few rows against weights no cache holds, padded copies, blocks for
    operands of 2 GiB and more, generic kernel."""
    import workloads as wl
    tn = hg.Layouts.make(b_col_major=True)
    for s in [wl.C1_SHAPE, *wl.C2_SHAPES, *wl.C3_SHAPES, *wl.C5_SHAPES, *wl.c4_shapes()[::7]]:
        assert hg.plan_choice(*s).startswith("table: "), s
        assert hg.plan_choice(*s, tn).startswith("table: "), s
    assert hg.plan_choice(16, 28672, 8192) == "table: skinny,sk=1"
    assert hg.plan_choice(1, 4096, 4096, tn).startswith("table: skinny,")        # column-major B has streaming rows of its own
    assert hg.plan_choice(1, 15360, 5120).startswith("table: skinny,") and hg.plan_choice(1, 15360, 5120, tn).startswith("table: mfma,")
    near = hg.plan_choice(3000, 5120, 5120)
    assert near.startswith("neighbour: mfma,bm=256,bn=256,") and "mi=16" in near
    assert hg.plan_choice(3000, 6144, 4096).startswith("model: mfma,bm=192,bn=192,")      # 512 tiles against the neighbour's 288
    assert hg.plan_choice(4096, 4096, 4096, hg.Layouts.make(lda=4104)).startswith(("neighbour: ", "model: "))   # not packed: no table row
    assert hg.plan_choice(8, 16384, 8192).startswith("model: skinny,")
    assert hg.plan_choice(8, 4096, 4096).startswith("model: mfma,")
    assert hg.plan_choice(300, 264, 128).startswith("model: mfma,")
    assert hg.plan_choice(1000, 1001, 1003).endswith(",pad=1")
    assert hg.plan_choice(100, 100, 100) == "generic" and hg.plan_choice(0, 5, 5) == "empty"
    assert hg.plan_choice(32768, 32768, 32768) == "blocks,rows=16384,cols=16384,bt=1"
    assert hg.plan_choice(32768, 32768, 32768, tn) == "blocks,rows=16384,cols=16384"
    assert hg.plan_choice((1 << 21), 64, 1024) == "blocks,rows=699136,cols=64"
    with pytest.raises(hg.HgemmError):
        hg.plan_choice(-1, 8, 8)
    with pytest.raises(hg.HgemmError):
        hg.plan_choice(64, 64, 64, hg.Layouts.make(lda=8))
