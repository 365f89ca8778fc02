"""Pins for the CPU oracle: every check here compares the oracle with something
that does not go through its own arithmetic -- numpy's float16, exact rational
brute force, closed forms, integer matmul, values the paper states."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import hgemm_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_kv(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                out[k] = v
    return out


# ---------------------------------------------------------------------------
# fp16 <-> fp64 conversion
# ---------------------------------------------------------------------------

def test_half_to_double_all_65536_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    got = orc.half_bits_to_double(bits)
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint64), want[~nan].view(np.uint64))  # includes -0.0 and subnormals
    assert np.array_equal(np.signbit(got), np.signbit(want))


def test_double_to_half_round_trip_all_finite_and_inf():
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    keep = ~np.isnan(vals)
    back = orc.double_to_half_bits(vals[keep])
    assert np.array_equal(back, bits[keep])


def _positive_finite_halves():
    bits = np.arange(0x0000, 0x7c00, dtype=np.uint16)      # +0 .. largest finite
    return bits, bits.view(np.float16).astype(np.float64)


def test_double_to_half_ties_go_to_even_at_every_midpoint():
    bits, vals = _positive_finite_halves()
    mid = (vals[:-1] + vals[1:]) / 2.0                      # exact in fp64
    lo_bits, hi_bits = bits[:-1], bits[1:]
    want_tie = np.where(lo_bits % 2 == 0, lo_bits, hi_bits)
    assert np.array_equal(orc.double_to_half_bits(mid), want_tie)
    # one fp64 ulp either side of the tie must leave the tie rule
    assert np.array_equal(orc.double_to_half_bits(np.nextafter(mid, 0.0)), lo_bits)
    assert np.array_equal(orc.double_to_half_bits(np.nextafter(mid, np.inf)), hi_bits)
    # same on the negative side (sign symmetric)
    assert np.array_equal(orc.double_to_half_bits(-mid), want_tie | 0x8000)
    # numpy's own conversion is an independent implementation of the same rounding
    assert np.array_equal(mid.astype(np.float16).view(np.uint16), want_tie)


def test_double_to_half_edges():
    f = orc.double_to_half_bits
    assert f([65504.0])[0] == 0x7BFF
    assert f([65519.99])[0] == 0x7BFF
    assert f([65520.0])[0] == 0x7C00                      # tie between 65504 and 2^16 -> even -> overflow
    assert f([-65520.0])[0] == 0xFC00
    assert f([1e300])[0] == 0x7C00
    assert f([2.0 ** -24])[0] == 0x0001                   # smallest subnormal
    assert f([2.0 ** -25])[0] == 0x0000                   # tie with zero -> even -> zero
    assert f([np.nextafter(2.0 ** -25, 1.0)])[0] == 0x0001
    assert f([3 * 2.0 ** -25])[0] == 0x0002               # tie between 1 and 2 units -> even
    assert f([2.0 ** -14 - 2.0 ** -25])[0] == 0x0400      # largest subnormal + half unit -> ties to even -> smallest normal
    assert f([0.0])[0] == 0x0000
    assert f([-0.0])[0] == 0x8000
    assert f([np.inf])[0] == 0x7C00
    nanbits = int(f([np.nan])[0])
    assert (nanbits & 0x7C00) == 0x7C00 and (nanbits & 0x3FF) != 0
    # a value that rounding via fp32 first would get wrong (double rounding):
    # 1 + 2^-11 + 2^-30 is above the tie, so it must round up to 1 + 2^-10
    x = 1.0 + 2.0 ** -11 + 2.0 ** -30
    assert f([x])[0] == 0x3C01
    assert np.float32(x).astype(np.float16).view(np.uint16) == 0x3C00   # the trap the oracle avoids


def test_double_to_half_random_matches_numpy():
    rng = np.random.default_rng(123)
    parts = [
        rng.standard_normal(200_000) * 100.0,
        rng.standard_normal(200_000) * 1e-4,               # subnormal range
        rng.standard_normal(100_000) * 1e-7,               # below the smallest subnormal
        rng.standard_normal(100_000) * 4e4,                # overflow range
        rng.uniform(-2048, 2048, 200_000),
    ]
    x = np.concatenate(parts)
    assert np.array_equal(orc.double_to_half_bits(x), x.astype(np.float16).view(np.uint16))


# ---------------------------------------------------------------------------
# the product: exact rational brute force on tiny shapes
# ---------------------------------------------------------------------------

def _all_finite_halves_as_fractions():
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16)
    finite = np.isfinite(vals)
    pos = (bits < 0x7C00)
    b = bits[finite & pos]
    return b, [Fraction(float(v)) for v in vals[finite & pos].astype(np.float64)]


_POS_BITS, _POS_FRACS = _all_finite_halves_as_fractions()


def _round_fraction_to_half_bits(q: Fraction) -> int:
    """Nearest-even rounding of an exact rational to fp16, by search over the
    table of all non-negative finite fp16 values.  Independent of the oracle."""
    sign = 0x8000 if q < 0 else 0
    a = abs(q)
    top = _POS_FRACS[-1]
    if a >= top + (top - _POS_FRACS[-2]) / 2:              # >= 65520 overflows
        return sign | 0x7C00
    lo, hi = 0, len(_POS_FRACS) - 1
    while hi - lo > 1:
        mid = (lo + hi) // 2
        if _POS_FRACS[mid] <= a:
            lo = mid
        else:
            hi = mid
    if a >= top:
        return sign | int(_POS_BITS[-1])
    dl, dh = a - _POS_FRACS[lo], _POS_FRACS[hi] - a
    if dl < dh:
        pick = lo
    elif dh < dl:
        pick = hi
    else:
        pick = lo if int(_POS_BITS[lo]) % 2 == 0 else hi
    return sign | int(_POS_BITS[pick])


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (2, 3, 5), (3, 2, 8), (5, 5, 3), (8, 1, 2), (1, 8, 5), (3, 5, 1)])
@pytest.mark.parametrize("seed", [0, 1])
def test_brute_force_exact_rational_tiny_shapes(M, N, K, seed):
    rng = np.random.default_rng([seed, M, N, K])
    A = (rng.standard_normal((M, K)) * 3).astype(np.float16)
    B = (rng.standard_normal((K, N)) * 3).astype(np.float16)
    got = orc.hgemm(A, B).view(np.uint16)
    for i in range(M):
        for j in range(N):
            q = sum((Fraction(float(A[i, k])) * Fraction(float(B[k, j])) for k in range(K)), Fraction(0))
            assert int(got[i, j]) == _round_fraction_to_half_bits(q), (i, j)


def test_brute_force_with_subnormals_and_large_values():
    # mixes fp16 subnormals, tiny normals and values near the top of the range;
    # K is small enough that the fp64 sum is exact.
    vals = np.array([6e-8, -6e-8, 3e-5, 6.1e-5, 1.0, -0.333, 255.0, 1000.0, -2047.0, 60000.0 / 1024], dtype=np.float16)
    rng = np.random.default_rng(5)
    A = rng.choice(vals, size=(4, 3))
    B = rng.choice(vals, size=(3, 4))
    got = orc.hgemm(A, B).view(np.uint16)
    for i in range(4):
        for j in range(4):
            q = sum((Fraction(float(A[i, k])) * Fraction(float(B[k, j])) for k in range(3)), Fraction(0))
            assert int(got[i, j]) == _round_fraction_to_half_bits(q)


def test_overflow_and_nan_semantics():
    A = np.array([[60000.0, 60000.0]], dtype=np.float16)
    B = np.array([[1.0], [1.0]], dtype=np.float16)
    assert orc.hgemm(A, B).view(np.uint16)[0, 0] == 0x7C00          # 120000 -> +inf
    assert orc.hgemm(-A, B).view(np.uint16)[0, 0] == 0xFC00
    A2 = np.array([[np.nan, 1.0]], dtype=np.float16)
    assert np.isnan(orc.hgemm(A2, B)[0, 0])
    A3 = np.array([[np.inf, -np.inf]], dtype=np.float16)
    assert np.isnan(orc.hgemm(A3, B)[0, 0])                         # inf - inf


# ---------------------------------------------------------------------------
# structure: identity, zero, permutation, single-one, transposition traps
# ---------------------------------------------------------------------------

def test_identity_zero_permutation():
    rng = np.random.default_rng(9)
    B = rng.standard_normal((7, 11)).astype(np.float16)
    I = np.eye(7, dtype=np.float16)
    assert np.array_equal(orc.hgemm(I, B).view(np.uint16), B.view(np.uint16))
    A = rng.standard_normal((5, 7)).astype(np.float16)
    assert np.array_equal(orc.hgemm(A, np.eye(7, dtype=np.float16)).view(np.uint16), A.view(np.uint16))
    Z = np.zeros((5, 7), dtype=np.float16)
    assert np.array_equal(orc.hgemm(Z, B), np.zeros((5, 11), dtype=np.float16))
    perm = rng.permutation(7)
    P = np.zeros((7, 7), dtype=np.float16)
    P[np.arange(7), perm] = 1                                       # row i of P*B is row perm[i] of B
    assert np.array_equal(orc.hgemm(P, B).view(np.uint16), B[perm].view(np.uint16))


def test_single_one_selects_one_row_and_one_column():
    rng = np.random.default_rng(10)
    B = rng.standard_normal((6, 9)).astype(np.float16)
    A = np.zeros((4, 6), dtype=np.float16)
    A[2, 5] = 1                                                     # C[2,:] = B[5,:], other rows zero
    C = orc.hgemm(A, B)
    assert np.array_equal(C[2].view(np.uint16), B[5].view(np.uint16))
    assert not C[[0, 1, 3]].any()
    A = rng.standard_normal((4, 6)).astype(np.float16)
    E = np.zeros((6, 9), dtype=np.float16)
    E[1, 7] = 1                                                     # C[:,7] = A[:,1]
    C = orc.hgemm(A, E)
    assert np.array_equal(C[:, 7].view(np.uint16), A[:, 1].view(np.uint16))
    assert not np.delete(C, 7, axis=1).any()


def test_non_square_integer_matmul_matches_int64():
    # distinct M, N, K and non-symmetric values: a transposed operand, swapped
    # leading dimension or dropped k term cannot survive this.
    rng = np.random.default_rng(11)
    for (M, N, K) in [(3, 5, 7), (17, 9, 33), (64, 48, 100), (1, 130, 257), (129, 1, 64)]:
        Ai = rng.integers(-3, 4, size=(M, K))
        Bi = rng.integers(-3, 4, size=(K, N))
        want = (Ai.astype(np.int64) @ Bi.astype(np.int64))
        assert np.abs(want).max() <= 2048
        got = orc.hgemm(Ai.astype(np.float16), Bi.astype(np.float16)).astype(np.int64)
        assert np.array_equal(got, want)


def test_closed_forms():
    thr = int(_golden_kv("paper_exactness_thresholds.txt")["integer_exact_below"])
    for K in (1, 64, 1000, 2047, thr):
        A = np.ones((3, K), dtype=np.float16)
        B = np.ones((K, 4), dtype=np.float16)
        assert np.array_equal(orc.hgemm(A, B).astype(np.int64), np.full((3, 4), K))
    K = 300
    A = np.ones((2, K), dtype=np.float16)
    B = np.tile(((np.arange(10) % 5) - 2).astype(np.float16), (K, 1))
    want = np.tile(K * ((np.arange(10) % 5) - 2), (2, 1))
    assert np.array_equal(orc.hgemm(A, B).astype(np.int64), want)
    # rank-1: (u v^T) from K = 1
    u = np.arange(-4, 5).astype(np.float16).reshape(-1, 1)
    v = np.arange(1, 8).astype(np.float16).reshape(1, -1)
    assert np.array_equal(orc.hgemm(u, v).astype(np.int64), np.arange(-4, 5).reshape(-1, 1) * np.arange(1, 8))


def test_tn_layout_is_the_same_product():
    rng = np.random.default_rng(12)
    A = rng.standard_normal((9, 20)).astype(np.float16)
    B = rng.standard_normal((20, 13)).astype(np.float16)
    nn = orc.hgemm(A, B)
    tn = orc.hgemm(A, np.ascontiguousarray(B.T), b_col_major=True)
    assert np.array_equal(nn.view(np.uint16), tn.view(np.uint16))


def test_sampled_entry_points_agree_with_full_and_with_rationals():
    rng = np.random.default_rng(13)
    A = rng.standard_normal((12, 31)).astype(np.float16)
    B = rng.standard_normal((31, 10)).astype(np.float16)
    C = orc.hgemm(A, B)
    ii = np.array([0, 11, 5, 5, 3])
    jj = np.array([0, 9, 2, 7, 9])
    assert np.array_equal(orc.hgemm_at(A, B, ii, jj).view(np.uint16), C[ii, jj].view(np.uint16))
    sums = orc.hgemm_sum_at(A, B, ii, jj)
    for t in range(len(ii)):
        q = sum((Fraction(float(A[ii[t], k])) * Fraction(float(B[k, jj[t]])) for k in range(31)), Fraction(0))
        assert abs(Fraction(float(sums[t])) - q) <= abs(q) * Fraction(1, 2 ** 45) + Fraction(1, 2 ** 60)
    with pytest.raises(RuntimeError):
        orc.hgemm_at(A, B, np.array([12]), np.array([0]))


def test_empty_shapes():
    A = np.zeros((0, 5), dtype=np.float16)
    B = np.zeros((5, 3), dtype=np.float16)
    assert orc.hgemm(A, B).shape == (0, 3)
    A = np.zeros((2, 0), dtype=np.float16)
    B = np.zeros((0, 3), dtype=np.float16)
    assert np.array_equal(orc.hgemm(A, B), np.zeros((2, 3), dtype=np.float16))   # empty sum is +0


# ---------------------------------------------------------------------------
# real-valued inputs: independent library routines
# ---------------------------------------------------------------------------

def test_matches_numpy_float64_matmul_rounded_once():
    rng = np.random.default_rng(14)
    for (M, N, K) in [(64, 80, 96), (33, 17, 512)]:
        A = rng.uniform(-1, 1, (M, K)).astype(np.float16)
        B = rng.uniform(-1, 1, (K, N)).astype(np.float16)
        want = (A.astype(np.float64) @ B.astype(np.float64)).astype(np.float16)
        got = orc.hgemm(A, B)
        diff = int((got.view(np.uint16) != want.view(np.uint16)).sum())
        # a different fp64 summation order can only flip a result that sits
        # within ~1e-13 of a rounding tie; none is expected in a few thousand values
        assert diff == 0


def test_paper_eq1_fp32_reference_within_one_ulp():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(15)
    A = rng.uniform(-1, 1, (48, 256)).astype(np.float16)
    B = rng.uniform(-1, 1, (256, 40)).astype(np.float16)
    ref32 = torch.matmul(torch.from_numpy(A).float(), torch.from_numpy(B).float()).numpy()
    got = orc.hgemm(A, B).astype(np.float64)
    ulp = np.spacing(np.abs(got).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(got - ref32.astype(np.float64)) <= ulp)


# ---------------------------------------------------------------------------
# the paper's exactness statements (Section 2.3.2 and footnotes)
# ---------------------------------------------------------------------------

def test_binary_inputs_exact_below_2048_even_with_fp16_partial_sums():
    thr = int(_golden_kv("paper_exactness_thresholds.txt")["integer_exact_below"])
    rng = np.random.default_rng(16)
    K = 4096
    # P(product = 1) = 0.5: the sums scatter around K/2 = 2048, so both sides of the threshold occur
    p = 0.5 ** 0.5
    A = (rng.random((6, K)) < p).astype(np.float16)
    B = (rng.random((K, 6)) < p).astype(np.float16)
    ref = orc.hgemm(A, B).astype(np.float64)
    exact = A.astype(np.int64) @ B.astype(np.int64)
    below = exact < thr
    assert below.any() and (~below).any()
    assert np.array_equal(ref[below], exact[below].astype(np.float64))
    # sequential fp16 accumulation (what an fp16-accumulate kernel would do):
    # monotone partial sums stay exact wherever the final value is below 2048
    acc = np.zeros((6, 6), dtype=np.float16)
    for k in range(K):
        acc = (acc + np.outer(A[:, k], B[k, :]).astype(np.float16)).astype(np.float16)
    assert np.array_equal(acc[below].astype(np.int64), exact[below])


def test_half_integer_threshold_is_1024():
    thr = int(_golden_kv("paper_exactness_thresholds.txt")["half_integer_exact_below"])
    ones = np.ones((1, thr), dtype=np.float16)

    def row_sum(n_ones, n_halves):
        a = np.concatenate([np.ones(n_ones), np.full(n_halves, 0.5)]).astype(np.float16).reshape(1, -1)
        b = np.ones((a.shape[1], 1), dtype=np.float16)
        return float(orc.hgemm(a, b)[0, 0])

    assert row_sum(thr - 1, 1) == thr - 0.5          # 1023.5 is representable
    assert row_sum(thr, 1) == float(thr)             # 1024.5 -> tie -> even -> 1024
    assert row_sum(thr + 1, 1) == float(thr + 2)     # 1025.5 -> tie -> even -> 1026
    assert float(orc.hgemm(ones, ones.T.copy())[0, 0]) == float(thr)


def test_signed_inputs_can_break_fp16_accumulation_but_not_the_oracle():
    # footnote of Section 2.3.2: with {-1,0,1} an fp16 running sum may pass 2048
    # and lose exactness before cancelling back; the fp64 oracle is unaffected.
    assert _golden_kv("paper_exactness_thresholds.txt")["signed_partial_sums_monotone"] == "no"
    a = np.concatenate([np.ones(2049), -np.ones(2049)]).astype(np.float16).reshape(1, -1)   # prefix reaches 2049
    b = np.ones((a.shape[1], 1), dtype=np.float16)
    assert float(orc.hgemm(a, b)[0, 0]) == 0.0
    acc = np.float16(0)
    for v in a[0]:
        acc = np.float16(acc + v)
    assert float(acc) != 0.0                         # 2048 + 1 is not representable: the running sum sticks


# ---------------------------------------------------------------------------
# planted mistakes: each plausible slip must be caught by the pins above
# ---------------------------------------------------------------------------

def _mutants():
    def transposed_b(A, B):
        return orc.hgemm(A, np.ascontiguousarray(B.T)) if B.shape[0] == B.shape[1] else None

    def dropped_last_k(A, B):
        return orc.hgemm(A[:, :-1], B[:-1, :])

    def via_fp32_rounding(A, B):
        s = A.astype(np.float64) @ B.astype(np.float64)
        return s.astype(np.float32).astype(np.float16)

    def fp16_products(A, B):
        p = (A[:, :, None].astype(np.float16) * B[None, :, :].astype(np.float16)).astype(np.float16)
        return p.astype(np.float64).sum(axis=1).astype(np.float16)

    return {"transposed_b": transposed_b, "dropped_last_k": dropped_last_k,
            "via_fp32_rounding": via_fp32_rounding, "fp16_products": fp16_products}


@pytest.mark.parametrize("name", sorted(_mutants()))
def test_pins_catch_planted_mistakes(name):
    mutant = _mutants()[name]
    rng = np.random.default_rng(17)
    caught = False
    # pin 1: integer matmul on non-symmetric square inputs
    Ai = rng.integers(-3, 4, size=(16, 16))
    Bi = rng.integers(-3, 4, size=(16, 16))
    out = mutant(Ai.astype(np.float16), Bi.astype(np.float16))
    if out is not None and not np.array_equal(out.astype(np.int64), Ai @ Bi):
        caught = True
    # pin 2: fp64 matmul rounded once, on real inputs including a constructed near-tie
    A = rng.uniform(-1, 1, (32, 64)).astype(np.float16)
    B = rng.uniform(-1, 1, (64, 32)).astype(np.float16)
    A[0, :] = 0
    B[:, 0] = 0
    A[0, 0], A[0, 1], A[0, 2] = 1.0, 2.0 ** -11, 2.0 ** -14       # 1 + 2^-11 + 2^-24*... just above a tie
    B[0, 0], B[1, 0], B[2, 0] = 1.0, 1.0, 2.0 ** -10
    want = (A.astype(np.float64) @ B.astype(np.float64)).astype(np.float16)
    out = mutant(A, B)
    if out is not None and not np.array_equal(out.view(np.uint16), want.view(np.uint16)):
        caught = True
    assert caught, f"no pin notices the planted mistake {name!r}"
    # and the real oracle passes both
    assert np.array_equal(orc.hgemm(Ai.astype(np.float16), Bi.astype(np.float16)).astype(np.int64), Ai @ Bi)
    assert np.array_equal(orc.hgemm(A, B).view(np.uint16), want.view(np.uint16))


# ---------------------------------------------------------------------------
# the 16-bit accumulator variant (Section 1: fp16 accumulators are a valid choice for fp16 inputs;
# Section 2.3.2: the exact-match test keeps every output at or below 2048 for their sake)
# ---------------------------------------------------------------------------

def _acc16_by_hand(A, B, block):
    """Independent emulation: exact block sums in int64 units of 2^-6 (inputs are multiples of 1/8), the running
    value rounded to fp16 by numpy's own float64 -> float16 cast after every block."""
    Ai = np.rint(A.astype(np.float64) * 8).astype(np.int64)
    Bi = np.rint(B.astype(np.float64) * 8).astype(np.int64)
    M, K = Ai.shape
    N = Bi.shape[1]
    acc = np.zeros((M, N), dtype=np.float16)
    for k0 in range(0, K, block):
        s = Ai[:, k0:k0 + block] @ Bi[k0:k0 + block, :]                       # exact
        acc = (acc.astype(np.float64) + s.astype(np.float64) / 64.0).astype(np.float16)
    return acc


@pytest.mark.parametrize("block", [1, 3, 16, 32])
@pytest.mark.parametrize("M,N,K", [(3, 4, 40), (2, 5, 16), (4, 3, 97), (1, 1, 1), (5, 2, 33)])
def test_acc16_matches_an_independent_emulation_on_exactly_representable_inputs(M, N, K, block):
    rng = np.random.default_rng(1000 * K + block)
    A = (rng.integers(-32, 33, size=(M, K)) / 8.0).astype(np.float16)       # multiples of 1/8, |x| <= 4
    B = (rng.integers(-32, 33, size=(K, N)) / 8.0).astype(np.float16)
    want = _acc16_by_hand(A, B, block)
    got = orc.hgemm_acc16(A, B, block)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))
    ii, jj = np.divmod(np.arange(M * N), N)
    assert np.array_equal(orc.hgemm_acc16_at(A, B, ii, jj, block).view(np.uint16), want.ravel().view(np.uint16))
    assert np.array_equal(orc.hgemm_acc16(A, np.ascontiguousarray(B.T), block, b_col_major=True).view(np.uint16), want.view(np.uint16))


def test_acc16_paper_exact_match_property_binary_inputs_up_to_2048():
    """Section 2.3.2: with inputs in {0, 1} every output is a count; an fp16 accumulator holds counts up to 2048
    exactly, whatever the cadence of its roundings."""
    rng = np.random.default_rng(5)
    K = 4000
    p = np.sqrt(0.45)                                                           # E[c] = 1800, max stays under 2048
    A = (rng.random((12, K)) < p).astype(np.float16)
    B = (rng.random((K, 9)) < p).astype(np.float16)
    exact = A.astype(np.int64) @ B.astype(np.int64)
    assert exact.max() <= 2048 and exact.min() > 1024
    for block in (1, 16, 64):
        assert np.array_equal(orc.hgemm_acc16(A, B, block).astype(np.int64), exact), block


def test_acc16_closed_forms_tell_the_cadences_apart():
    ones_a = np.ones((1, 70000), dtype=np.float16)
    ones_b = np.ones((70000, 1), dtype=np.float16)
    # one product at a time: 2048 + 1 ties to 2048 and the sum sticks there
    assert float(orc.hgemm_acc16(ones_a, ones_b, 1)[0, 0]) == 2048.0
    # 16 at a time: exact while multiples of 16 are representable, i.e. up to 32768; 32768 + 16 ties to 32768
    assert float(orc.hgemm_acc16(ones_a, ones_b, 16)[0, 0]) == 32768.0
    assert float(orc.hgemm_acc16(ones_a[:, :32768], ones_b[:32768], 16)[0, 0]) == 32768.0
    assert float(orc.hgemm_acc16(ones_a[:, :20000], ones_b[:20000], 16)[0, 0]) == 20000.0
    # 32 at a time: exact all the way to 65504 + 32 = 65536, which overflows to infinity
    assert np.isposinf(orc.hgemm_acc16(ones_a, ones_b, 32)[0, 0])
    # a ragged last block is not dropped: 40 = 16 + 16 + 8
    assert float(orc.hgemm_acc16(ones_a[:, :40], ones_b[:40], 16)[0, 0]) == 40.0
    # one block covering all of K is the fp64-accumulate definition
    assert float(orc.hgemm_acc16(ones_a[:, :40000], ones_b[:40000], 1 << 20)[0, 0]) == float(orc.hgemm(ones_a[:, :40000], ones_b[:40000])[0, 0]) == 40000.0


def test_acc16_with_k_within_one_block_is_the_definition_on_real_inputs():
    rng = np.random.default_rng(9)
    for K in (1, 7, 16):
        A = rng.standard_normal((9, K)).astype(np.float16)
        B = rng.standard_normal((K, 11)).astype(np.float16)
        assert np.array_equal(orc.hgemm_acc16(A, B, 16).view(np.uint16), orc.hgemm(A, B).view(np.uint16))
    A = rng.standard_normal((6, 200)).astype(np.float16)
    B = rng.standard_normal((200, 5)).astype(np.float16)
    assert np.array_equal(orc.hgemm_acc16(A, B, 200).view(np.uint16), orc.hgemm(A, B).view(np.uint16))
    # and with many blocks the error against the definition stays what fp16 accumulation allows (a few ulp of the
    # running sum per block), far inside the parity tolerance
    got = orc.hgemm_acc16(A, B, 16).astype(np.float64)
    ref = orc.hgemm(A, B).astype(np.float64)
    assert np.all(np.abs(got - ref) <= 1e-2 * np.maximum(1.0, np.abs(ref)))
    assert not np.array_equal(got, ref)


def test_acc16_rejects_bad_arguments_and_handles_empty_shapes():
    a = np.ones((2, 3), dtype=np.float16)
    b = np.ones((3, 2), dtype=np.float16)
    with pytest.raises(RuntimeError):
        orc.hgemm_acc16(a, b, 0)
    assert orc.hgemm_acc16(np.ones((0, 3), np.float16), b, 16).shape == (0, 2)
    assert np.array_equal(orc.hgemm_acc16(np.ones((2, 0), np.float16), np.ones((0, 2), np.float16), 16), np.zeros((2, 2), np.float16))
