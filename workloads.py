"""Seeded synthetic inputs for the HGEMM workloads.

This module only draws random numbers and lists shapes.  It holds none of the
method's arithmetic (no products, no sums, no rounding decisions of the GEMM)
and is the one piece shared by the CPU oracle's tests and the GPU path's tests
and benchmark.  Every generator returns numpy ``float16`` arrays: the fp16
values ARE the inputs, for both sides.

Workloads (the paper's evaluation uses random inputs over a grid of (M,N,K)
triples, Abstract and Section 2.3.2; the concrete recipes are this build's):

  C1  single 256^3, entries uniform[-1,1], seed 0
  C2  square sweep n^3, n in {1024,2048,4096,8192}, entries N(0,1)/sqrt(K)
  C3  LLM-projection skinny shapes, A ~ N(0,1), B ~ N(0, 0.02^2)
  C4  200 triples drawn with seed 1 from {64,...,12288}^3, entries uniform[-1,1]
  C5  16384 x 16384 x {8192,16384} uniform[-1,1], and a small-integer variant

Draws are made in float32, one row block at a time (so a 16384^2 operand never
needs more than a block of wide temporaries), and rounded once to fp16 by numpy.
"""
from __future__ import annotations

import math
from typing import Iterator, List, Sequence, Tuple

import numpy as np

Shape = Tuple[int, int, int]

GRID_VALUES: Tuple[int, ...] = (64, 128, 256, 512, 1024, 2048, 4096, 8192, 12288)
PAPER_GRID_VALUES: Tuple[int, ...] = GRID_VALUES + (16384,)   # the paper's 10-value grid (Abstract)

C1_SHAPE: Shape = (256, 256, 256)
C2_SHAPES: Tuple[Shape, ...] = tuple((n, n, n) for n in (1024, 2048, 4096, 8192))
C3_M: Tuple[int, ...] = (1, 16, 64, 128, 512)
C3_NK: Tuple[Tuple[int, int], ...] = ((4096, 4096), (11008, 4096), (4096, 11008), (14336, 4096))
C3_SHAPES: Tuple[Shape, ...] = tuple((m, n, k) for (n, k) in C3_NK for m in C3_M)
# Not one of the five configurations: the same kind of shape for a model four times the size (hidden
# width 8192, feed-forward width 28672), inputs by the C3 recipe.  Weights of 128-448 MiB show what
# the memory-bound kernels reach when launch and ramp-up no longer weigh on a 10-20 us call.
C3_LARGE_M: Tuple[int, ...] = (1, 16, 64)
C3_LARGE_NK: Tuple[Tuple[int, int], ...] = ((8192, 8192), (28672, 8192), (8192, 28672))
C3_LARGE_SHAPES: Tuple[Shape, ...] = tuple((m, n, k) for (n, k) in C3_LARGE_NK for m in C3_LARGE_M)
# Also outside the five configurations: projections of other common model widths (hidden 5120 with
# feed-forward 13824 and a fused 3 x 5120 attention projection; grouped-query attention projections of
# 6144 x 4096 and 10240 x 8192), C3's token counts and input recipe.  They are in the dispatch table so
# that a user of such a model gets measured choices rather than modelled ones.
C3_OTHER_NK: Tuple[Tuple[int, int], ...] = ((5120, 5120), (13824, 5120), (5120, 13824), (15360, 5120), (6144, 4096), (10240, 8192))
C3_OTHER_SHAPES: Tuple[Shape, ...] = tuple((m, n, k) for (n, k) in C3_OTHER_NK for m in C3_M)
C5_SHAPES: Tuple[Shape, ...] = ((16384, 16384, 8192), (16384, 16384, 16384))
C5_INT_SHAPE: Shape = (16384, 16384, 128)

_ROW_BLOCK = 1024


def _rng(config_id: int, shape: Shape, extra: int = 0) -> np.random.Generator:
    M, N, K = shape
    return np.random.default_rng(np.random.SeedSequence([config_id, M, N, K, extra]))


def _fill(rows: int, cols: int, draw) -> np.ndarray:
    """Fill a (rows, cols) float16 array block by block; ``draw(r, c)`` returns float32."""
    out = np.empty((rows, cols), dtype=np.float16)
    for r0 in range(0, rows, _ROW_BLOCK):
        r1 = min(rows, r0 + _ROW_BLOCK)
        out[r0:r1] = draw(r1 - r0, cols).astype(np.float16)
    return out


def uniform_pm1(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """iid uniform on [-1, 1)."""
    return _fill(rows, cols, lambda r, c: rng.random((r, c), dtype=np.float32) * np.float32(2) - np.float32(1))


def normal(rng: np.random.Generator, rows: int, cols: int, std: float) -> np.ndarray:
    """iid N(0, std^2)."""
    s = np.float32(std)
    return _fill(rows, cols, lambda r, c: rng.standard_normal((r, c), dtype=np.float32) * s)


def integers(rng: np.random.Generator, rows: int, cols: int, lo: int, hi: int) -> np.ndarray:
    """iid uniform over the integers lo..hi inclusive (all exactly representable in fp16)."""
    return _fill(rows, cols, lambda r, c: rng.integers(lo, hi + 1, size=(r, c), dtype=np.int8).astype(np.float32))


def bernoulli(rng: np.random.Generator, rows: int, cols: int, p: float, value: float = 1.0) -> np.ndarray:
    """Entries ``value`` with probability p, else 0."""
    v = np.float32(value)
    return _fill(rows, cols, lambda r, c: (rng.random((r, c), dtype=np.float32) < np.float32(p)).astype(np.float32) * v)


# ---- the five workload configurations ------------------------------------------------

def c1_inputs() -> Tuple[np.ndarray, np.ndarray]:
    M, N, K = C1_SHAPE
    rng = np.random.default_rng(0)
    return uniform_pm1(rng, M, K), uniform_pm1(rng, K, N)


def c2_inputs(shape: Shape) -> Tuple[np.ndarray, np.ndarray]:
    M, N, K = shape
    rng = _rng(2, shape)
    s = 1.0 / math.sqrt(K)
    return normal(rng, M, K, s), normal(rng, K, N, s)


def c3_inputs(shape: Shape) -> Tuple[np.ndarray, np.ndarray]:
    M, N, K = shape
    rng = _rng(3, shape)
    return normal(rng, M, K, 1.0), normal(rng, K, N, 0.02)


def c4_shapes(count: int = 200, seed: int = 1) -> List[Shape]:
    """``count`` distinct triples from GRID_VALUES^3, in draw order (seed 1)."""
    n = len(GRID_VALUES)
    idx = np.random.default_rng(seed).choice(n ** 3, size=count, replace=False)
    out = []
    for t in idx.tolist():
        m, rest = divmod(t, n * n)
        nn, k = divmod(rest, n)
        out.append((GRID_VALUES[m], GRID_VALUES[nn], GRID_VALUES[k]))
    return out


def c4_inputs(shape: Shape) -> Tuple[np.ndarray, np.ndarray]:
    M, N, K = shape
    rng = _rng(4, shape)
    return uniform_pm1(rng, M, K), uniform_pm1(rng, K, N)


def c5_inputs(shape: Shape) -> Tuple[np.ndarray, np.ndarray]:
    M, N, K = shape
    rng = _rng(5, shape)
    return uniform_pm1(rng, M, K), uniform_pm1(rng, K, N)


# ---- exact-answer families (Section 2.3.2, "Exact Match with binary Inputs") ---------

def small_int_inputs(shape: Shape, seed: int = 0, lo: int = -2, hi: int = 2) -> Tuple[np.ndarray, np.ndarray]:
    """Signed small integers.  With fp32 accumulation every partial sum is an
    exact integer as long as it stays below 2^24, whatever the summation order."""
    M, N, K = shape
    rng = _rng(6, shape, seed)
    return integers(rng, M, K, lo, hi), integers(rng, K, N, lo, hi)


def binary_inputs(shape: Shape, seed: int = 0, value: float = 1.0, target: float = 1024.0
                  ) -> Tuple[np.ndarray, np.ndarray]:
    """Entries in {0, value}; P(value) chosen so that the expected count of
    non-zero products per output element is about ``target`` (or K if smaller)."""
    M, N, K = shape
    p = min(1.0, math.sqrt(target / K)) if K > 0 else 1.0
    rng = _rng(7, shape, seed)
    return bernoulli(rng, M, K, p, value), bernoulli(rng, K, N, p, 1.0)


def exact_family_for(shape: Shape, seed: int = 0) -> Tuple[str, np.ndarray, np.ndarray]:
    """Pick an integer family whose products are exactly representable in
    fp16 for this K: {-2..2} while 4K <= 2048, {-1,0,1} while K <= 2048, else binary."""
    M, N, K = shape
    if 4 * K <= 2048:
        a, b = small_int_inputs(shape, seed, -2, 2)
        return "int[-2,2]", a, b
    if K <= 2048:
        a, b = small_int_inputs(shape, seed, -1, 1)
        return "int[-1,1]", a, b
    a, b = binary_inputs(shape, seed)
    return "binary", a, b


def sample_positions(shape: Shape, count: int, seed: int = 0, tile: int = 256
                     ) -> Tuple[np.ndarray, np.ndarray]:
    """Positions (i, j) for a sampled comparison on a large output: the four
    corners, points on both sides of tile boundaries, and uniform random ones."""
    M, N, _ = shape
    rng = np.random.default_rng(np.random.SeedSequence([8, M, N, seed]))
    rows = {0, min(1, M - 1), M - 1}
    cols = {0, min(1, N - 1), N - 1}
    for t in range(tile, M, tile):
        if len(rows) < 64:
            rows.update((t - 1, t))
    for t in range(tile, N, tile):
        if len(cols) < 64:
            cols.update((t - 1, t))
    rows = np.array(sorted(rows), dtype=np.int64)
    cols = np.array(sorted(cols), dtype=np.int64)
    gi, gj = np.meshgrid(rows, cols, indexing="ij")
    ii = [gi.ravel()]
    jj = [gj.ravel()]
    rest = max(0, count - ii[0].size)
    ii.append(rng.integers(0, M, size=rest, dtype=np.int64))
    jj.append(rng.integers(0, N, size=rest, dtype=np.int64))
    return np.concatenate(ii), np.concatenate(jj)


# ---- the same distributions drawn on the device (timing runs only) --------------------

def device_inputs(config: str, shape: Shape, device: str = "cuda"):
    """(A, B) as fp16 torch tensors on ``device`` with the distribution of workload ``config``
    ("C1".."C5"), drawn by torch's seeded generator there.  For timing runs, where a few hundred
    operand sets would take minutes to draw on the host and the values only matter through their
    distribution; the parity tests always use the numpy generators above, whose arrays both sides read."""
    import torch

    M, N, K = shape
    gen = torch.Generator(device=device)
    gen.manual_seed((int(config[1:]) * 1000003 + M) * 1000003 + N * 1009 + K)

    def uniform(r, c):
        return (torch.rand((r, c), device=device, generator=gen) * 2 - 1).half()

    def gauss(r, c, std):
        return (torch.randn((r, c), device=device, generator=gen) * std).half()

    if config == "C2":
        s = 1.0 / math.sqrt(K)
        return gauss(M, K, s), gauss(K, N, s)
    if config == "C3":
        return gauss(M, K, 1.0), gauss(K, N, 0.02)
    if config in ("C1", "C4", "C5"):
        return uniform(M, K), uniform(K, N)
    raise ValueError(config)


def all_bench_shapes() -> Iterator[Tuple[str, Shape]]:
    yield "C1", C1_SHAPE
    for s in C2_SHAPES:
        yield "C2", s
    for s in C3_SHAPES:
        yield "C3", s
    for s in c4_shapes():
        yield "C4", s
    for s in C5_SHAPES:
        yield "C5", s
