"""Helpers for the GPU parity tests: move numpy fp16 arrays through the C ABI and back."""
import numpy as np
import torch

import paper_2512_02551_amd as hg

TOL = 1e-2          # elementwise |C - C_ref| <= TOL * max(1, |C_ref|) on real-valued inputs


def to_dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda().view(torch.float16)


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.float16)


def run_hgemm(a: np.ndarray, b: np.ndarray, spec=None, b_col_major=False, prefill=float("nan"), guard=0):
    """C = A @ B through hgemm_plan(_override) / hgemm_run.  C (and, with ``guard`` > 0, a band of
    ``guard`` extra rows before and after it) is pre-filled with ``prefill`` so leaks of old
    contents show up.  Returns (C, band_before, band_after, description)."""
    M, K = a.shape
    N = b.shape[0] if b_col_major else b.shape[1]
    da, db = to_dev(a), to_dev(b)
    cols = max(N, 1)
    full = torch.full((M + 2 * guard, cols), prefill, dtype=torch.float16, device="cuda")
    c = full[guard:guard + M]
    lay = hg.Layouts.make(b_col_major=b_col_major)
    with hg.Plan(M, N, K, lay, spec) as p:
        desc = p.describe()
        p.run(da.data_ptr(), db.data_ptr(), c.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    out = to_host(full)
    return out[guard:guard + M, :N], out[:guard], out[guard + M:], desc


def assert_close(c: np.ndarray, ref: np.ndarray, what=""):
    c64, r64 = c.astype(np.float64), ref.astype(np.float64)
    assert np.array_equal(np.isnan(c64), np.isnan(r64)), f"{what}: NaN masks differ"
    # an overflow (or its absence) must agree, sign included, before the finite values are compared
    assert np.array_equal(np.isinf(c64), np.isinf(r64)), f"{what}: infinity masks differ"
    inf = np.isinf(r64)
    assert np.array_equal(np.sign(c64[inf]), np.sign(r64[inf])), f"{what}: infinities of opposite sign"
    ok = ~np.isnan(r64) & ~inf
    err = np.abs(c64[ok] - r64[ok])
    bound = TOL * np.maximum(1.0, np.abs(r64[ok]))
    bad = err > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} elements outside tolerance, worst {float((err / bound).max()):.3g}x bound"


def assert_bit_exact(c: np.ndarray, ref: np.ndarray, what=""):
    diff = c.view(np.uint16) != ref.view(np.uint16)
    # +0 and -0 are the same number; an exact integer result is never -0 on either side, but be explicit
    diff &= ~((c == 0) & (ref == 0))
    if diff.any():
        idx = np.argwhere(diff)[:5]
        detail = ", ".join(f"[{i},{j}] got {float(c[i, j])} want {float(ref[i, j])}" for i, j in idx)
        raise AssertionError(f"{what}: {int(diff.sum())} elements differ: {detail}")
