"""hgemm_run_static, the entry point that allocates nothing: its output must equal hgemm_plan + hgemm_run's
bit for bit (same kernels, the workspace in the library's static scratch array instead of an allocation),
on calls in a row that reuse the scratch, the later ones smaller; problems beyond the scratch are refused."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2512_02551_amd as hg  # noqa: E402
import workloads as wl  # noqa: E402
from oracle import hgemm_oracle as orc  # noqa: E402

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import assert_bit_exact, assert_close, run_hgemm, to_dev, to_host  # noqa: E402


def _run_static(a, b, b_col_major=False, prefill=float("nan")):
    M, K = a.shape
    N = b.shape[0] if b_col_major else b.shape[1]
    da, db = to_dev(a), to_dev(b)
    full = torch.full((M + 2, max(N, 1)), prefill, dtype=torch.float16, device="cuda")
    c = full[1:1 + M]
    import gc
    gc.collect()
    before = torch.cuda.memory_allocated()
    hg.run_static(M, N, K, hg.Layouts.make(b_col_major=b_col_major), da.data_ptr(), db.data_ptr(), c.data_ptr(),
                  torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() <= before      # nothing was taken from torch's allocator either
    out = to_host(full)
    assert np.isnan(out[0]).all() and np.isnan(out[-1]).all(), "wrote outside C"
    return out[1:1 + M, :N]


def test_static_entry_point_matches_planned_run_on_calls_in_a_row():
    # split-K plans (fp32 planes in the scratch), the second smaller than the first so that it finds the
    # first one's partial sums in the scratch; then an unaligned shape (padded copies in the scratch), a
    # plan that needs no workspace, and the first shape again
    shapes = [(64, 4096, 11008), (16, 4096, 4096), (100, 1001, 1003), (512, 512, 512), (64, 4096, 11008)]
    uses_workspace = 0
    for shape in shapes:
        M, N, K = shape
        name, a, b = wl.exact_family_for(shape, seed=41)
        want, _, _, desc = run_hgemm(a, b)
        with hg.Plan(M, N, K) as p:
            uses_workspace += p.workspace_bytes() > 0
            assert p.workspace_bytes() <= hg.STATIC_SCRATCH_BYTES
        got = _run_static(a, b)
        assert_bit_exact(got, want, f"static {shape} {name} {desc}")
        # and against the oracle on real inputs
        rng = np.random.default_rng([M, N, K, 5])
        a = wl.uniform_pm1(rng, M, K)
        b = wl.uniform_pm1(rng, K, N)
        want, _, _, _ = run_hgemm(a, b)
        got = _run_static(a, b)
        assert_bit_exact(got, want, f"static real {shape} {desc}")
        ii, jj = wl.sample_positions(shape, 1500, seed=6)
        ref = orc.hgemm_at(a, b, ii, jj).astype(np.float64)
        err = np.abs(got[ii, jj].astype(np.float64) - ref)
        assert (err <= 1e-2 * np.maximum(1.0, np.abs(ref))).all()
    assert uses_workspace >= 3


def test_static_entry_point_tn_layout_and_degenerate_sizes():
    shape = (48, 2048, 8192)
    name, a, b = wl.exact_family_for(shape, seed=42)
    bt = np.ascontiguousarray(b.T)
    want, _, _, desc = run_hgemm(a, bt, b_col_major=True)
    assert_bit_exact(_run_static(a, bt, b_col_major=True), want, f"static TN {desc}")
    # K = 0 gives zeros; M = 0 and N = 0 launch nothing
    z = _run_static(np.zeros((5, 0), np.float16), np.zeros((0, 24), np.float16))
    assert z.shape == (5, 24) and (z == 0).all()
    hg.run_static(0, 8, 8, None, 0, 0, 0, torch.cuda.current_stream().cuda_stream)
    hg.run_static(8, 0, 8, None, 0, 0, 0, torch.cuda.current_stream().cuda_stream)


def test_static_entry_point_on_rows_of_the_streaming_family():
    # table rows that name the streaming family: fused reduction (arrival counters in the scratch, which must come
    # back to zero for the next call), two-launch reduction (planes in the scratch), and the column-major kernel
    for (shape, tn) in [((1, 8192, 8192), False), ((16, 8192, 8192), False), ((1, 8192, 8192), False), ((1, 4096, 4096), True)]:
        M, N, K = shape
        assert hg.plan_choice(M, N, K, hg.Layouts.make(b_col_major=tn)).startswith("table: skinny,")
        name, a, b = wl.exact_family_for(shape, seed=43)
        bb = np.ascontiguousarray(b.T) if tn else b
        want, _, _, desc = run_hgemm(a, bb, b_col_major=tn)
        assert desc.startswith("skinny,")
        assert_bit_exact(_run_static(a, bb, b_col_major=tn), want, f"static {shape} {name} {desc}")
        ii, jj = wl.sample_positions(shape, 1000, seed=7)
        ref = orc.hgemm_at(a, b, ii, jj)
        sel = np.abs(ref.astype(np.float64)) <= 2048
        assert np.array_equal(want[ii, jj][sel].astype(np.float64), ref[sel].astype(np.float64)), desc


def test_static_entry_point_refuses_what_does_not_fit():
    # a split-K plan whose planes exceed the static scratch: refused with a status of its own, nothing launched
    M, N, K = 2048, 2048, 16384
    with hg.Plan(M, N, K) as p:
        need = p.workspace_bytes()
    c = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    a = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    b = torch.zeros((K, N), dtype=torch.float16, device="cuda")
    if need > hg.STATIC_SCRATCH_BYTES:
        with pytest.raises(hg.HgemmError) as e:
            hg.run_static(M, N, K, None, a.data_ptr(), b.data_ptr(), c.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert e.value.status == hg.ERR_WORKSPACE
        torch.cuda.synchronize()
        assert torch.isnan(c).all()
    # unaligned and large: the padded copies alone exceed the scratch
    M, N, K = 4096, 4097, 4096
    a = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    b = torch.zeros((K, N), dtype=torch.float16, device="cuda")
    c = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    with pytest.raises(hg.HgemmError) as e:
        hg.run_static(M, N, K, None, a.data_ptr(), b.data_ptr(), c.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert e.value.status == hg.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert torch.isnan(c).all()
    with pytest.raises(hg.HgemmError):
        hg.run_static(-1, 8, 8, None, 0, 0, 0, 0)
