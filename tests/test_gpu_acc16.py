"""GPU parity of the 16-bit accumulator variant ("ac=16" specs) against the oracle's acc16 variant.

Section 1 of the paper names fp16 accumulators as a valid choice for fp16 inputs and Section 2.3.2 builds its
exact-match test for them ({0,1} inputs, outputs kept at or below 2048).  Here the running sums are rounded to fp16
after every matrix-core instruction, i.e. after every 16 products; on integer inputs every intermediate is exact
before its rounding on both sides, so the comparison is bit for bit even where the roundings bite."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2512_02551_amd as hg  # noqa: E402
from oracle import hgemm_oracle as orc  # noqa: E402

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import assert_bit_exact, run_hgemm  # noqa: E402


def acc16_specs():
    out = []
    for line in hg.spec_help().splitlines():
        if "compiled" in line:
            for tup in line.split(":")[1].split():
                bm, bn, bk, wm, wn, st, pf = (int(x) for x in tup.strip("()").split(","))
                out.append(f"mfma,bm={bm},bn={bn},bk={bk},wm={wm},wn={wn},st={st},pf={pf},sk=1,gm=8,ac=16")
    assert out
    return out


def assert_within_two_ulps_of_the_running_sum(c, ref, a, b, what):
    """Tolerance of the 16-bit accumulator on real inputs.  The matrix-core instruction adds its 16 products to the
    accumulator in fp32, the oracle in fp64; where the sum before a rounding sits within 2^-24 of a tie the two fall to
    different fp16 neighbours, and from there on the running sums differ by one fp16 ulp of their magnitude at that
    point (about one output in a hundred at K = 2000).  Bound: two fp16 ulps (2^-9 relative) of the largest running
    sum of that output, computed here in fp64 block by block."""
    acc = np.zeros(ref.shape, dtype=np.float64)
    biggest = np.ones(ref.shape, dtype=np.float64)
    for k0 in range(0, a.shape[1], 16):
        acc += a[:, k0:k0 + 16].astype(np.float64) @ b[k0:k0 + 16, :].astype(np.float64)
        biggest = np.maximum(biggest, np.abs(acc))
    c64, r64 = c.astype(np.float64), ref.astype(np.float64)
    assert np.array_equal(np.isnan(c64), np.isnan(r64)), f"{what}: NaN masks differ"
    assert np.array_equal(np.isinf(c64), np.isinf(r64)), f"{what}: infinity masks differ"
    ok = np.isfinite(r64)
    err = np.abs(c64[ok] - r64[ok])
    bound = 2.0 ** -9 * biggest[ok]
    assert not (err > bound).any(), f"{what}: {int((err > bound).sum())} elements outside two ulps of the running sum, worst {float((err / bound).max()):.3g}x"
    # and the two sides agree exactly almost everywhere
    assert (err == 0).mean() > 0.9, f"{what}: only {float((err == 0).mean()):.3f} of the elements agree exactly"


def small_counts(shape, seed, hi=4):
    M, N, K = shape
    rng = np.random.default_rng(seed)
    return rng.integers(0, hi, size=(M, K)).astype(np.float16), rng.integers(0, hi, size=(K, N)).astype(np.float16)


@pytest.mark.parametrize("shape", [(72, 136, 1096), (300, 264, 1000)])
def test_every_spec_rounds_like_the_oracle_where_sums_pass_2048(shape):
    """Inputs in {0..3}: outputs average 2.25 K > 2048, so the fp16 running sum rounds on the way (spacing 2, then 4),
    and K = 1000 ends in a block of 8.  Every compiled configuration must reproduce the oracle bit for bit."""
    a, b = small_counts(shape, seed=shape[2])
    ref = orc.hgemm_acc16(a, b, 16)
    exact = a.astype(np.int64) @ b.astype(np.int64)
    assert exact.max() > 2048 and (ref.astype(np.int64) != exact).any()          # the roundings do bite
    for spec in acc16_specs():
        c, before, after, desc = run_hgemm(a, b, spec=spec, guard=2)
        assert desc.endswith("ac=16"), desc
        assert_bit_exact(c, ref, desc)
        assert np.isnan(before).all() and np.isnan(after).all(), desc


def test_every_spec_tn_layout_and_the_papers_exact_match_property():
    """Section 2.3.2: {0,1} inputs with every output at or below 2048 come out exact with an fp16 accumulator."""
    shape = (96, 200, 4000)
    rng = np.random.default_rng(3)
    p = np.sqrt(0.45)
    a = (rng.random((shape[0], shape[2])) < p).astype(np.float16)
    b = (rng.random((shape[2], shape[1])) < p).astype(np.float16)
    exact = a.astype(np.int64) @ b.astype(np.int64)
    assert exact.max() <= 2048
    ref = orc.hgemm_acc16(a, b, 16)
    assert np.array_equal(ref.astype(np.int64), exact)
    bt = np.ascontiguousarray(b.T)
    for spec in acc16_specs()[::3]:
        c, _, _, desc = run_hgemm(a, b, spec=spec)
        assert_bit_exact(c, ref, desc)
        c, _, _, desc = run_hgemm(a, bt, spec=spec, b_col_major=True)
        assert_bit_exact(c, ref, "TN " + desc)


def test_closed_form_sum_of_ones_sticks_at_32768():
    """Sixteen ones at a time: exact up to 32768, where adding 16 ties back to 32768 (an fp32 accumulator gives 40000,
    which overflows fp16 only above 65504)."""
    a = np.ones((32, 40000), dtype=np.float16)
    b = np.ones((40000, 64), dtype=np.float16)
    c, _, _, desc = run_hgemm(a, b, spec="mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=1,gm=8,ac=16")
    assert (c == 32768.0).all(), desc
    c32, _, _, _ = run_hgemm(a, b, spec="mfma,bm=32,bn=64,bk=64,wm=1,wn=2,st=4,pf=3,sk=1,gm=8")
    assert (c32.astype(np.float64) == 40000.0).all()


def test_real_inputs_within_tolerance_deterministic_and_special_values():
    shape = (200, 264, 2056)
    rng = np.random.default_rng(11)
    a = rng.uniform(-1, 1, (shape[0], shape[2])).astype(np.float16)
    b = rng.uniform(-1, 1, (shape[2], shape[1])).astype(np.float16)
    ref = orc.hgemm_acc16(a, b, 16)
    for spec in ("mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=3,sk=1,gm=8,ac=16", "mfma,bm=128,bn=128,bk=64,wm=2,wn=2,st=3,pf=3,sk=1,gm=8,ac=16",
                 "mfma,bm=256,bn=256,bk=64,wm=2,wn=4,st=2,pf=1,sk=1,gm=8,ac=16"):
        c1, _, _, desc = run_hgemm(a, b, spec=spec)
        c2, _, _, _ = run_hgemm(a, b, spec=spec)
        assert_within_two_ulps_of_the_running_sum(c1, ref, a, b, desc)
        assert np.array_equal(c1.view(np.uint16), c2.view(np.uint16)), desc
    # overflow of the running sum is sticky, NaN propagates
    a2 = a.copy()
    b2 = b.copy()
    a2[0, :] = 60.0
    b2[:, 0] = 60.0                     # 3600 per product: passes 65520 after two blocks
    a2[1, 5] = np.nan
    ref2 = orc.hgemm_acc16(a2, b2, 16)
    assert np.isposinf(ref2[0, 0]) and np.isnan(ref2[1]).all()
    c, _, _, desc = run_hgemm(a2, b2, spec="mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=3,sk=1,gm=8,ac=16")
    assert np.isposinf(c[0, 0]) and np.isnan(c[1]).all(), desc
    rest = np.ones(c.shape, dtype=bool)
    rest[0, 0] = False
    rest[1, :] = False
    rows = np.flatnonzero(rest.any(axis=1))
    assert_within_two_ulps_of_the_running_sum(c[rows][:, 1:], ref2[rows][:, 1:], a2[rows], b2[:, 1:], desc)


def test_only_explicit_whole_k_specs_get_the_16_bit_accumulator():
    base = "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=3"
    for bad in (base + ",sk=2,gm=8,ac=16", base + ",sk=1,gm=8,sm=1,ac=16", base + ",sk=1,gm=8,ps=1,ac=16", base + ",sk=1,gm=8,ac=8",
                "skinny,sk=4,ac=16"):
        with pytest.raises(hg.HgemmError):
            hg.Plan(64, 256, 4096, None, bad)
    for shape in ((256, 256, 256), (64, 4096, 4096), (4096, 4096, 4096), (1000, 1001, 1003)):
        with hg.Plan(*shape) as p:
            assert "ac=16" not in p.describe()
    assert all("ac=16" not in c for c in hg.candidates(512, 512, 512))
