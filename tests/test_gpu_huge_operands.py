"""Operands of 2 GiB and more lie beyond the 32-bit buffer offsets of the matrix-core kernels: hgemm_plan runs such
problems as a grid of blocks (row blocks of A and C, column panels of B and C; a row-major B of that size goes
through a transposed copy first).  The operands here are periodic repetitions of small seeded integer blocks, so the
oracle can rebuild any row of A and any column of B from the blocks and evaluate sampled rows / columns of C."""
import re

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2512_02551_amd as hg  # noqa: E402
import workloads as wl  # noqa: E402
from oracle import hgemm_oracle as orc  # noqa: E402

pytestmark = pytest.mark.gpu

if torch.cuda.is_available():
    from gpu_util import assert_bit_exact, to_dev, to_host  # noqa: E402

GIB2 = 1 << 31


def _tiled(block: np.ndarray, rows: int, cols: int) -> "torch.Tensor":
    """Device matrix rows x cols whose element (i, j) is block[i % R][j % C]."""
    R, C = block.shape
    t = to_dev(block).repeat(-(-rows // R), -(-cols // C))
    return t[:rows, :cols].contiguous()


def _edges(n: int, step: int, rng, extra: int):
    """Indices at both ends, on both sides of every multiple of `step`, and a few random ones."""
    idx = {0, 1, n - 2, n - 1}
    for b in range(step, n, step):
        idx.update({b - 1, b, b + 1})
    idx.update(int(x) for x in rng.integers(0, n, size=extra))
    return np.array(sorted(i for i in idx if 0 <= i < n))


def test_tall_a_of_more_than_2_gib_runs_in_row_blocks():
    M, N, K = (1 << 20) + 300, 264, 1024
    assert M * K * 2 >= GIB2
    rng = np.random.default_rng(101)
    block = wl.integers(rng, 4099, K, -2, 2)          # A[m] = block[m % 4099]
    b = wl.integers(rng, K, N, -2, 2)
    da, db = _tiled(block, M, K), to_dev(b)
    c = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    with hg.Plan(M, N, K) as p:
        desc = p.describe()
        assert desc.startswith("blocks,") and "bt=1" not in desc, desc
        rows_per_block = int(re.search(r"rows=(\d+)", desc).group(1))
        assert rows_per_block < M and (rows_per_block + 512) * K * 2 < GIB2
        p.run(da.data_ptr(), db.data_ptr(), c.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    assert not bool(torch.isnan(c).any()), "part of C was not written"
    ii = _edges(M, rows_per_block, rng, 150)
    ref = orc.hgemm(block[ii % block.shape[0]], b)
    assert_bit_exact(to_host(c[torch.from_numpy(ii).cuda()]), ref, f"{M}x{N}x{K} {desc}")


@pytest.mark.parametrize("b_col_major", [False, True], ids=["row-major B", "column-major B"])
def test_b_of_more_than_2_gib_runs_in_column_panels(b_col_major):
    M, N, K = 264, 32768 + 512, 32768
    assert K * N * 2 >= GIB2
    rng = np.random.default_rng(102 + int(b_col_major))
    a = wl.integers(rng, M, K, -2, 2)
    block = wl.integers(rng, 1021, 1031, -2, 2)       # B[k][n] = block[k % 1021][n % 1031]
    if b_col_major:
        db = _tiled(np.ascontiguousarray(block.T), N, K)     # stored N x K
    else:
        db = _tiled(block, K, N)
    da = to_dev(a)
    c = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    with hg.Plan(M, N, K, hg.Layouts.make(b_col_major=b_col_major)) as p:
        desc = p.describe()
        assert desc.startswith("blocks,") and (("bt=1" in desc) != b_col_major), desc
        cols_per_panel = int(re.search(r"cols=(\d+)", desc).group(1))
        assert cols_per_panel < N and (cols_per_panel + 512) * K * 2 < GIB2
        for call in range(2):                 # the transposed copy is rewritten by every call
            c.fill_(float("nan"))
            p.run(da.data_ptr(), db.data_ptr(), c.data_ptr(), torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            assert not bool(torch.isnan(c).any()), "part of C was not written"
            jj = _edges(N, cols_per_panel, rng, 120)
            b_cols = block[np.arange(K) % block.shape[0]][:, jj % block.shape[1]]
            ref = orc.hgemm(a, np.ascontiguousarray(b_cols))
            assert_bit_exact(to_host(c[:, torch.from_numpy(jj).cuda()]), ref, f"{M}x{N}x{K} {desc} call {call}")


def test_blocked_plans_are_not_for_the_entry_point_that_allocates_nothing_and_explicit_specs_refuse():
    M, N, K = (1 << 20) + 300, 64, 1024
    with pytest.raises(hg.HgemmError):
        hg.Plan(M, N, K, None, "mfma,bm=64,bn=64,bk=64,wm=2,wn=2,st=4,pf=3,sk=1,gm=8")
    with hg.Plan(M, N, K) as p:
        assert p.describe().startswith("blocks,")
        assert p.workspace_bytes() >= 0
