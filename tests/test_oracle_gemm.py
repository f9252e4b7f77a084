"""Pins for slice products, recomposition, the exact reference and the whole oracle call
(O6-O8): integer matrices reproduce an int64 matmul exactly, the componentwise bound against
exact rationals, brute-force sufficiency of the ESC-chosen slice count, routing."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import exact as ex
from oracle import ozaki as oz
from paper_2511_13778_amd import workloads as wl


def test_k_block_rule():
    assert oz.k_block_length(7) == 18432
    assert oz.k_block_length(9) == 14336
    for S in range(1, oz.MAX_SLICES + 1):
        kb = oz.k_block_length(S)
        assert kb % 256 == 0 and kb > 0
        # worst anti-diagonal plus the largest carry from below fits int32
        assert S * kb * 128 * 128 + (1 << 23) < 2 ** 31
        assert S * (kb + 256) * 128 * 128 + (1 << 23) >= 2 ** 31 or S * (kb + 256) > (1 << 17) - (1 << 9) - 1


def test_products_match_literal_loops():
    rng = np.random.default_rng(1)
    As = rng.integers(-128, 128, (4, 5, 13)).astype(np.int8)
    Bs = rng.integers(-128, 128, (4, 3, 13)).astype(np.int8)
    np.testing.assert_array_equal(oz.slice_products(As, Bs), oz.slice_products_loops(As, Bs))


def test_products_extreme_digits_fit_int32():
    S = 3
    k = oz.k_block_length(S) + 300                   # two k-blocks
    As = np.full((S, 2, k), -128, dtype=np.int8)
    Bs = np.full((S, 2, k), -128, dtype=np.int8)
    P = oz.slice_products(As, Bs)
    assert P.shape == (2, S, 2, 2)
    assert P[0, 2, 0, 0] == 3 * oz.k_block_length(S) * 16384
    assert P[1, 0, 1, 1] == 300 * 16384


def test_integer_matrices_are_exact():
    # integers below 2^21 with a full-size entry in every row/column: only the three leading
    # digits are non-zero, so no slice pair is dropped and nothing is truncated; the emulated
    # product must equal the textbook integer product bit for bit.
    rng = np.random.default_rng(2)
    m, k, n = 17, 50, 11
    A = rng.integers(-(2 ** 21) + 1, 2 ** 21, (m, k)).astype(np.float64)
    B = rng.integers(-(2 ** 21) + 1, 2 ** 21, (k, n)).astype(np.float64)
    A[:, 0] = 2 ** 20 + 3
    B[0, :] = -(2 ** 20) - 5
    want = A.astype(np.int64) @ B.astype(np.int64)
    tr = oz.emulated_dgemm(A, B, mode=oz.MODE_FIXED_UNGUARDED, max_bits=55)
    assert tr.verdict.slices_used == 7
    assert np.all(tr.As[3:] == 0) and np.all(tr.Bs[3:] == 0)
    np.testing.assert_array_equal(tr.C, want.astype(np.float64))
    # a transposed operand or a swapped index must break this
    assert not np.array_equal(tr.C[:n, :n], (B.T.astype(np.int64)[:, :k] @ A.T.astype(np.int64)[:k, :])[:n, :n].astype(np.float64))


def test_recompose_weights():
    # one k-block, S = 3, a single entry: P_d contributes P_d * 256^-d * 2^(eA+eB-10)
    P = np.zeros((1, 3, 1, 1), dtype=np.int32)
    P[0, :, 0, 0] = (5, -7, 11)
    got = oz.recompose(P, np.array([4]), np.array([-3]))
    assert got[0, 0] == (5 - 7 / 256 + 11 / 65536) * 2.0 ** (4 - 3 - 10)
    # two k-blocks add in the unscaled range
    P2 = np.concatenate([P, P], axis=0)
    assert oz.recompose(P2, np.array([4]), np.array([-3]))[0, 0] == 2 * got[0, 0]


def _exact_Z(P, kb, i, j):
    S = P.shape[1]
    return sum(int(P[kb, d, i, j]) * 256 ** (S - 1 - d) for d in range(S))


@pytest.mark.parametrize("S", [1, 2, 3, 7, 8, 12, 26])
def test_normalised_digits_are_the_exact_integer(S):
    # the carry-normalised digits are balanced base-256 digits of the exact integer sum_d P_d 256^(S-1-d)
    # under a signed leading word: same value, every lower digit in [-128, 127], and a small
    # integer stays small in every digit
    rng = np.random.default_rng(S)
    bound = ((1 << 17) - (1 << 9) - 1) << 14             # what the k-block rule admits for |P_d|
    P = rng.integers(-bound, bound + 1, (2, S, 3, 4)).astype(np.int32)
    P[0, :, 0, 0] = -bound                               # extremes of the admitted range
    P[0, :, 0, 1] = bound
    P[1, :, 1, 1] = 0
    P[1, :, 2, 2] = -1                                   # borrows ripple through every digit
    T0, lo = oz.normalised_digits(P)
    assert T0.dtype == np.int32 and lo.dtype == np.int8 and lo.shape == (2, S - 1, 3, 4)
    if S >= 2:                                           # -1 in every anti-diagonal: no borrow ripple
        assert T0[1, 2, 2] == -1 and np.all(lo[1, :, 2, 2] == -1)
    for kb in range(2):
        for i in range(3):
            for j in range(4):
                Z = int(T0[kb, i, j]) * 256 ** (S - 1) + sum(int(lo[kb, d - 1, i, j]) * 256 ** (S - 1 - d) for d in range(1, S))
                assert Z == _exact_Z(P, kb, i, j)


@pytest.mark.parametrize("S", [1, 2, 5, 7])
def test_recompose_is_the_exact_integer_rounded_once(S):
    # up to seven slices the FP64 recomposition of a k-block is the correctly rounded value of the
    # exact integer: no intermediate rounding, whatever the signs of the anti-diagonal sums
    rng = np.random.default_rng(40 + S)
    P = rng.integers(-(2 ** 30), 2 ** 30, (1, S, 6, 5)).astype(np.int32)
    eA, eB = rng.integers(-30, 30, 6), rng.integers(-30, 30, 5)
    got = oz.recompose(P, eA, eB)
    for i in range(6):
        for j in range(5):
            want = Fraction(_exact_Z(P, 0, i, j)) * Fraction(2) ** (int(eA[i] + eB[j]) + 2 * oz.H - 12 - 8 * (S - 1))
            assert got[i, j] == float(want)              # Fraction -> float rounds to nearest even


def test_recompose_many_slices_stays_within_an_ulp():
    rng = np.random.default_rng(9)
    P = rng.integers(-(2 ** 30), 2 ** 30, (3, 12, 4, 4)).astype(np.int32)
    z = np.zeros(4, dtype=np.int64)
    got = oz.recompose(P, z, z)
    for i in range(4):
        for j in range(4):
            want = sum(Fraction(_exact_Z(P, kb, i, j)) for kb in range(3)) * Fraction(2) ** (2 * oz.H - 12 - 88)
            assert abs(Fraction(float(got[i, j])) - want) <= 3 * abs(want) * Fraction(2) ** -52


def test_worst_case_digits_with_carry_fit_int32():
    # every digit at the extreme that makes all products positive, longest k-block: the aggregated
    # anti-diagonals (sum plus incoming carry) still fit the accumulator
    for S in (3, 7, 26):
        k = oz.k_block_length(S)
        As = np.full((S, 1, k), -128, dtype=np.int8)
        Bs = np.full((S, 1, k), -128, dtype=np.int8)
        P = oz.slice_products(As, Bs)
        T0, lo = oz.normalised_digits(P)                   # asserts the int32 range internally
        assert P[0, S - 1, 0, 0] == S * k * 16384


def test_fsum_reference_matches_rationals():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((4, 60)) * np.exp2(rng.integers(-40, 40, (4, 60)))
    B = rng.standard_normal((60, 3)) * np.exp2(rng.integers(-40, 40, (60, 3)))
    C = rng.standard_normal((4, 3))
    idx = [(i, j) for i in range(4) for j in range(3)]
    fr = ex.exact_gemm_fraction(A, B)
    got = ex.exact_entries(A, B, idx)
    assert all(got[t] == float(fr[i][j]) for t, (i, j) in enumerate(idx))
    fr2 = ex.exact_gemm_fraction(A, B, 1.5, 0.5, C)
    got2 = ex.exact_entries(A, B, idx, 1.5, 0.5, C)
    assert all(got2[t] == float(fr2[i][j]) for t, (i, j) in enumerate(idx))
    assert ex.exact_dot_fraction(A[1], B[:, 2]) == sum(
        (Fraction(float(a)) * Fraction(float(b)) for a, b in zip(A[1], B[:, 2])), Fraction(0))
    assert ex.exact_dot_fraction(np.array([5e-324, 3.0]), np.array([5e-324, -0.0])) == Fraction(5e-324) ** 2
    got3 = ex.exact_entries(A, B, idx, 1.0, 0.5, C)
    fr3 = ex.exact_gemm_fraction(A, B, 1.0, 0.5, C)
    assert all(got3[t] == float(fr3[i][j]) for t, (i, j) in enumerate(idx))


@pytest.mark.parametrize("gen,seed", [("pm1", 1), ("u01", 2), ("logn", 3)])
def test_55bit_mode_meets_componentwise_bound(gen, seed):
    m, k, n = 12, 96, 10
    if gen == "pm1":
        A, B = wl.uniform_pm1(m, k, n, seed)
    elif gen == "u01":
        A, B = wl.uniform_01(m, k, n, seed)
    else:
        A, B = wl.lognormal_spread(m, k, n, 0.5, seed)
    tr = oz.emulated_dgemm(A, B, mode=oz.MODE_FORCED_GUARDED, max_bits=55)
    assert tr.verdict.fallback == 0 and tr.verdict.slices_used == 7
    ratio = ex.gradeA_ratio(tr.C, ex.exact_gemm_fraction(A, B), ex.bound_denominator(A, B), k)
    assert ratio <= 1.0
    # a dropped anti-diagonal must be visible at this tolerance
    bad = oz.axpby(1.0, oz.recompose(tr.P[:, :6], tr.eA, tr.eB), 0.0, None)
    assert ex.gradeA_ratio(bad, ex.exact_gemm_fraction(A, B), ex.bound_denominator(A, B), k) > 1.0


def test_alpha_beta():
    A, B, C = wl.lognormal_spread(9, 64, 7, 1.0, 4, with_c=True)
    tr = oz.emulated_dgemm(A, B, 1.5, 0.5, C, mode=oz.MODE_DYNAMIC, max_bits=200)
    fr = ex.exact_gemm_fraction(A, B, 1.5, 0.5, C)
    den = ex.bound_denominator(A, B, None, 1.5, 0.5, C)
    assert ex.gradeA_ratio(tr.C, fr, den, 64) <= 1.0


def _min_slices_meeting_bound(A, B, k):
    fr = ex.exact_gemm_fraction(A, B)
    den = ex.bound_denominator(A, B)
    for S in range(1, oz.MAX_SLICES + 1):
        tr = oz.emulated_dgemm(A, B, mode=oz.MODE_FIXED_UNGUARDED, slices=S)
        if ex.gradeA_ratio(tr.C, fr, den, k) <= 1.0:
            return S
    return oz.MAX_SLICES + 1


@pytest.mark.parametrize("seed", range(24))
def test_esc_never_underestimates_slices(seed):
    # brute force on tiny cases: the smallest S that meets the bound against exact rationals
    # is never above the S the ESC route picks
    rng = np.random.default_rng(1000 + seed)
    m, k, n = int(rng.integers(1, 5)), int(rng.integers(1, 9)), int(rng.integers(1, 5))
    spread = int(rng.integers(0, 50))
    mant_bits = int(rng.choice([3, 12, 30, 53]))
    def draw(shape):
        v = rng.uniform(1, 2, shape) * rng.choice([-1, 1], shape)
        v = np.ldexp(np.round(np.ldexp(v, mant_bits - 1)), -(mant_bits - 1))   # few-bit significands
        return v * np.exp2(rng.integers(-spread, spread + 1, shape))
    A, B = draw((m, k)), draw((k, n))
    if seed % 4 == 0:
        A[rng.random((m, k)) < 0.3] = 0.0
    esc = oz.esc_coarse(A, B, int(rng.choice([1, 2, 4, 64])))
    assert esc >= oz.esc_exact(A, B)
    S_esc = oz.slices_dynamic(53, esc)
    if S_esc > oz.MAX_SLICES:
        pytest.skip("ESC route falls back")
    assert _min_slices_meeting_bound(A, B, k) <= S_esc


def test_wide_span_and_specials_route_to_fallback():
    A, B = wl.wide_span(8, 32, 8, 7)
    tr = oz.emulated_dgemm(A, B, mode=oz.MODE_DYNAMIC, max_bits=200)
    assert (tr.verdict.fallback, tr.verdict.reason) == (1, oz.REASON_BITS)
    assert tr.verdict.esc > 600
    A2, B2 = wl.plant_inf_nan(*wl.uniform_pm1(8, 32, 8, 8), seed=8)
    tr = oz.emulated_dgemm(A2, B2, mode=oz.MODE_DYNAMIC, max_bits=200)
    assert (tr.verdict.fallback, tr.verdict.reason, tr.verdict.infnan) == (1, oz.REASON_INFNAN, 1)


def test_rank1_cancellation_raises_slices_and_meets_bound():
    A, B = wl.rank1_cancel(10, 64, 6, 9)
    tr = oz.emulated_dgemm(A, B, mode=oz.MODE_DYNAMIC, max_bits=200)
    assert tr.verdict.fallback == 0 and tr.verdict.slices_used >= 8
    assert ex.gradeA_ratio(tr.C, ex.exact_gemm_fraction(A, B), ex.bound_denominator(A, B), 64) <= 1.0


def test_grading_test2_needs_guardrails():
    # with a fixed 55 bits the diagonal x^T x is lost once 2b+1 exceeds the bits; the guarded
    # variant falls back instead (aspect A1)
    A, B, x = wl.grading_test2(48, 40, 1)
    diag = float(sum(Fraction(float(v)) ** 2 for v in x))
    un = oz.emulated_dgemm(A, B, mode=oz.MODE_FIXED_UNGUARDED, max_bits=55)
    assert np.max(np.abs(np.diag(un.C) - diag) / diag) > 1e-6
    gd = oz.emulated_dgemm(A, B, mode=oz.MODE_FIXED_GUARDED, max_bits=55)
    assert (gd.verdict.fallback, gd.verdict.reason, gd.verdict.esc) == (1, oz.REASON_BITS, 81)
    assert np.max(np.abs(np.diag(gd.C) - diag) / diag) < 1e-13
    dyn = oz.emulated_dgemm(A, B, mode=oz.MODE_DYNAMIC, max_bits=200)
    assert dyn.verdict.slices_used == oz.slices_dynamic(53, 81)
    assert np.max(np.abs(np.diag(dyn.C) - diag) / diag) < 1e-14


def test_emergent_infinity_is_terminal_only():
    A = np.full((2, 4), 1.5e200)
    B = np.full((4, 2), 1.2e200)
    B[:, 1] *= -1
    tr = oz.emulated_dgemm(A, B, mode=oz.MODE_FORCED_GUARDED, max_bits=55)
    assert tr.verdict.fallback == 0
    assert np.all(tr.C[:, 0] == np.inf) and np.all(tr.C[:, 1] == -np.inf)
    # same magnitudes with cancellation stay finite: nothing overflows before the last step
    B2 = np.full((4, 2), 1.2e200)
    B2[::2] *= -1
    assert np.all(oz.emulated_dgemm(A, B2, mode=oz.MODE_FORCED_GUARDED).C == 0.0)


def test_degenerate_sizes_and_negative_zero():
    C = np.arange(6.0).reshape(2, 3)
    out = oz.emulated_dgemm(np.zeros((2, 0)), np.zeros((0, 3)), 1.0, 2.0, C).C
    np.testing.assert_array_equal(out, 2 * C)
    A = np.array([[-0.0, 1.0]])
    B = np.array([[5.0], [-0.0]])
    tr = oz.emulated_dgemm(A, B)
    assert tr.C[0, 0] == 0.0 and not np.signbit(tr.C[0, 0])
