"""Pins for the oracle's exponent scan, exact and coarsened ESC and the verdict (O1-O4)."""
import numpy as np
import pytest

from oracle import ozaki as oz
from paper_2511_13778_amd import workloads as wl


def test_exponents_true_ilogb():
    x = np.array([1.0, 1.999, 2.0, 0.5, -0.75, 5e-324, 2.0 ** -1060 * 1.5, 0.0, -0.0, 1.7e308])
    e = oz.exponents(x)
    assert list(e[:7]) == [0, 0, 1, -1, -1, -1074, -1060]
    assert e[7] == e[8] == oz.ZERO_EXP
    assert e[9] == 1023


def test_inf_nan_scan():
    x = np.ones((3, 3))
    assert not oz.has_inf_nan(x)
    for bad in (np.inf, -np.inf, np.nan):
        y = x.copy()
        y[1, 2] = bad
        assert oz.has_inf_nan(y)


def test_equal_exponents_give_one():
    rng = np.random.default_rng(0)
    A = rng.uniform(1, 2, (5, 9)) * rng.choice([-1, 1], (5, 9))
    B = rng.uniform(4, 8, (9, 4))
    assert oz.esc_exact(A, B) == 1
    for b in (1, 2, 4, 64):
        assert oz.esc_coarse(A, B, b) == 1


def test_hand_example():
    # row exponents (3, 0, -2), column exponents (-5, 1, 0): products 2^-2, 2^1, 2^-2
    A = np.array([[8.0, 1.0, 0.25]])
    B = np.array([[2.0 ** -5], [2.0], [1.0]])
    # eA = 3, eB = 1, z_r = 1  ->  3 + 1 - 1 + 1
    assert oz.esc_exact(A, B) == 4
    assert oz.esc_coarse(A, B, 1) == 4
    # one block: Max(x)+Min(y) = 3-5, Min(x)+Max(y) = -2+1  ->  zt = -1  ->  3+1+1+1
    assert oz.esc_coarse(A, B, 3) == 6


@pytest.mark.parametrize("nn,b", [(16, 3), (33, 10), (64, 40)])
def test_grading_test2_closed_form(nn, b):
    # diagonal dot products pair 2^j with 2^-j: eA = eB = b, best product exponent 0
    A, B, _ = wl.grading_test2(nn, b, seed=nn)
    assert oz.esc_exact(A, B) == 2 * b + 1
    for blk in (1, 4, 64):
        assert oz.esc_coarse(A, B, blk) == 2 * b + 1


def _random_pair(rng, m, k, n, spread, zeros):
    A = rng.standard_normal((m, k)) * np.exp2(rng.integers(-spread, spread + 1, (m, k)))
    B = rng.standard_normal((k, n)) * np.exp2(rng.integers(-spread, spread + 1, (k, n)))
    if zeros:
        A[rng.random((m, k)) < zeros] = 0.0
        B[rng.random((k, n)) < zeros] = 0.0
    return A, B


@pytest.mark.parametrize("seed", range(12))
def test_coarse_never_below_exact(seed):
    rng = np.random.default_rng(seed)
    m, k, n = rng.integers(1, 7), rng.integers(1, 40), rng.integers(1, 7)
    A, B = _random_pair(rng, m, k, n, spread=int(rng.integers(0, 30)), zeros=[0, 0.1, 0.5][seed % 3])
    ex = oz.esc_exact(A, B)
    assert oz.esc_coarse(A, B, 1) == ex
    prev = ex
    for b in (2, 4, 8, 16, 32, 64):                     # nested block sizes: monotone
        c = oz.esc_coarse(A, B, b)
        assert c >= prev
        prev = c


def test_zero_handling():
    A = np.array([[4.0, 0.0], [0.0, 0.0]])
    B = np.array([[1.0, 0.0], [0.5, 0.0]])
    # only pair (0,0) is live; its single non-zero product has exponent 2+0 = eA+eB
    assert oz.esc_exact(A, B) == 1
    assert oz.esc_coarse(A, B, 1) == 1
    # in one block Min(x) = -inf and Min(y) = 2^-1: candidates Max(x)+Min(y) = 2-1
    assert oz.esc_coarse(A, B, 2) == 2
    # every candidate -inf (a zero in each operand's only block): unbounded -> cap
    A2 = np.array([[4.0, 0.0]])
    B2 = np.array([[0.0], [1.0]])
    assert oz.esc_exact(A2, B2) == 1            # dot product is identically zero
    assert oz.esc_coarse(A2, B2, 2) == oz.ESC_CAP
    assert oz.esc_coarse(A2, B2, 1) == 1        # block view sees an all-zero side everywhere
    assert oz.esc_coarse(np.zeros((2, 2)), np.ones((2, 2)), 2) == 1
    # block-structured zeros: [A1 0] * [0; B2] is identically zero, needs no bits
    A3 = np.hstack([np.full((3, 4), 2.0 ** 20), np.zeros((3, 4))])
    B3 = np.vstack([np.zeros((4, 2)), np.full((4, 2), 2.0 ** -30)])
    assert oz.esc_coarse(A3, B3, 4) == 1
    assert oz.esc_coarse(A3, B3, 8) == oz.ESC_CAP


def test_scaling_invariance():
    rng = np.random.default_rng(3)
    A, B = _random_pair(rng, 5, 30, 4, spread=6, zeros=0)
    A2 = A * np.exp2(np.arange(5) * 3 - 4)[:, None]
    B2 = B * np.exp2(np.arange(4) * -5 + 2)[None, :]
    assert oz.esc_exact(A2, B2) == oz.esc_exact(A, B)
    assert oz.esc_coarse(A2, B2, 8) == oz.esc_coarse(A, B, 8)


def test_verdict_table():
    V = oz.verdict
    # forced: scan + ESC run, S from max_bits, only Inf/NaN falls back
    v = V(oz.MODE_FORCED_GUARDED, 53, 55, 0, False, 30, 64, 64, 64)
    assert (v.fallback, v.slices_used, v.esc, v.required_bits) == (0, 7, 30, 83)
    v = V(oz.MODE_FORCED_GUARDED, 53, 55, 0, True, -1, 64, 64, 64)
    assert (v.fallback, v.reason, v.infnan) == (1, oz.REASON_INFNAN, 1)
    # fixed + guard: falls back when target + ESC exceeds the available bits.  Seven slices carry
    # 8*7 - 2 = 54 magnitude bits (one headroom bit), so required_bits == max_bits == 55 is already
    # one bit more than they hold: the guard must trip exactly where the dynamic rule asks for 8
    assert V(oz.MODE_FIXED_GUARDED, 53, 55, 0, False, 1, 8, 8, 8).fallback == 0
    for esc in (2, 3):
        v = V(oz.MODE_FIXED_GUARDED, 53, 55, 0, False, esc, 8, 8, 8)
        assert (v.fallback, v.reason, v.required_bits) == (1, oz.REASON_BITS, 53 + esc)
    for mb in (39, 55, 63, 71):
        S = oz.slices_for_bits(mb)
        for esc in range(1, 30):
            v = V(oz.MODE_FIXED_GUARDED, 53, mb, 0, False, esc, 8, 8, 8)
            assert (v.fallback == 0) == (53 + esc <= mb and oz.slices_dynamic(53, esc) <= S)
            if not v.fallback:      # an accepted call never runs with fewer slices than the dynamic rule
                assert v.slices_used >= oz.slices_dynamic(53, esc)
    # an explicit slice count below what max_bits implies is held to the same capacity rule
    assert V(oz.MODE_FIXED_GUARDED, 20, 55, 4, False, 9, 8, 8, 8).fallback == 0      # 20 + 9 + 2 = 31 <= 32
    assert V(oz.MODE_FIXED_GUARDED, 20, 55, 4, False, 11, 8, 8, 8).fallback == 1     # 33 > 32
    # dynamic: S grows with ESC
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 1, 8, 8, 8).slices_used == 7
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 9, 8, 8, 8).slices_used == 8
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 17, 8, 8, 8).slices_used == 9
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 147, 8, 8, 8).slices_used == 26
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 148, 8, 8, 8).reason == oz.REASON_BITS
    # heuristic: tiny problems and huge slice counts go native
    hm = oz.HeuristicModel()
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 1, 32, 32, 32, hm).reason == oz.REASON_HEURISTIC
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 1, 8192, 8192, 8192, hm).fallback == 0
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 140, 8192, 8192, 8192, hm).reason == oz.REASON_HEURISTIC
    assert V(oz.MODE_FIXED_UNGUARDED, 53, 55, 0, False, -1, 8, 8, 8).slices_used == 7
    assert V(oz.MODE_FIXED_UNGUARDED, 53, 55, 9, False, -1, 8, 8, 8).slices_used == 9
    assert V(oz.MODE_NATIVE, 53, 55, 0, False, -1, 8, 8, 8).reason == oz.REASON_NATIVE


def test_shape_only_fallback_agrees_with_the_verdict():
    # the pre-check may only fire where the full verdict would say "heuristic" for every possible ESC
    hm = oz.HeuristicModel()
    for n in (16, 256, 1024, 3000, 4096, 8192):
        pre = oz.shape_only_fallback(oz.MODE_DYNAMIC, 53, n, n, n, hm)
        best = oz.verdict(oz.MODE_DYNAMIC, 53, 200, 0, False, 1, n, n, n, hm)       # ESC = 1: fewest slices
        assert pre == (best.reason == oz.REASON_HEURISTIC)
        if pre:
            for esc in (1, 5, 20, 60):
                assert oz.verdict(oz.MODE_DYNAMIC, 53, 200, 0, False, esc, n, n, n, hm).reason == oz.REASON_HEURISTIC
    assert oz.shape_only_fallback(oz.MODE_DYNAMIC, 53, 32, 32, 32, hm)
    assert not oz.shape_only_fallback(oz.MODE_DYNAMIC, 53, 8192, 8192, 8192, hm)
    assert not oz.shape_only_fallback(oz.MODE_DYNAMIC, 53, 32, 32, 32, None)          # heuristic off
    assert not oz.shape_only_fallback(oz.MODE_FORCED_GUARDED, 53, 32, 32, 32, hm)   # other modes never
    A = np.ones((8, 8)); A[0, 0] = np.inf
    tr = oz.emulated_dgemm(A, np.ones((8, 8)), mode=oz.MODE_DYNAMIC, max_bits=200, heuristic=hm)
    assert (tr.verdict.fallback, tr.verdict.reason, tr.verdict.esc, tr.verdict.infnan) == (1, oz.REASON_HEURISTIC, -1, 0)
