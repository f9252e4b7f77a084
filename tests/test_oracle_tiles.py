"""Pins for the oracle's per-tile slice counts (every TILE x TILE block of C takes the slice count of
its own ESC) and for the run-time heuristic's cost model.  Nothing here calls the HIP library."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import exact as ex
from oracle import ozaki as oz


def _structured(rng, m, k, n, wide_rows, spread):
    """Entries with nearly uniform exponents, except: each row i in `wide_rows` of A is one entry of
    normal size at a position l0 and 2^-spread times that elsewhere, and the entry of B that meets the
    large one is 2^-spread times the rest of its column in the first column and every third one.  Only
    those dot products have a large exponent span, so only the blocks of C that hold one need many bits."""
    A = rng.uniform(1, 2, (m, k)) * rng.choice([-1, 1], (m, k))
    B = rng.uniform(1, 2, (k, n)) * rng.choice([-1, 1], (k, n))
    for i in wide_rows:
        l0 = int(rng.integers(k))
        keep = A[i, l0]
        A[i] = np.ldexp(A[i], -spread)
        A[i, l0] = keep
        B[l0, ::3] = np.ldexp(B[l0, ::3], -spread)
    return A, B


@pytest.mark.parametrize("seed", range(6))
def test_tile_esc_is_the_esc_of_the_sub_product(seed):
    # a tile's rows of A and columns of B are whole rows and columns, so its ESC is the ESC of
    # that smaller product; the ESC of the whole product is the largest tile ESC
    rng = np.random.default_rng(seed)
    m, k, n, tile = int(rng.integers(3, 12)), int(rng.integers(4, 40)), int(rng.integers(3, 12)), int(rng.integers(2, 5))
    A, B = _structured(rng, m, k, n, [int(rng.integers(m))], 30)
    if seed % 2:
        A[rng.random(A.shape) < 0.1] = 0.0
    b = int(rng.choice([1, 4, 16]))
    T = oz.esc_coarse_tiles(A, B, b, tile)
    assert T.shape == (-(-m // tile), -(-n // tile))
    assert int(T.max()) == oz.esc_coarse(A, B, b)
    for ti in range(T.shape[0]):
        for tj in range(T.shape[1]):
            r, c = slice(ti * tile, (ti + 1) * tile), slice(tj * tile, (tj + 1) * tile)
            assert T[ti, tj] == oz.esc_coarse(A[r], B[:, c], b)
            assert T[ti, tj] >= oz.esc_exact(A[r], B[:, c])           # conservative tile by tile
    T1 = oz.esc_coarse_tiles(A, B, 1, tile)                            # b = 1: the exact ESC of each tile
    for ti in range(T.shape[0]):
        for tj in range(T.shape[1]):
            r, c = slice(ti * tile, (ti + 1) * tile), slice(tj * tile, (tj + 1) * tile)
            assert T1[ti, tj] == oz.esc_exact(A[r], B[:, c])


@pytest.mark.parametrize("S,Sp", [(3, 1), (5, 2), (7, 6), (9, 7), (12, 8), (26, 7)])
def test_leading_digits_of_a_longer_decomposition(S, Sp):
    # the first S' digits of the S-slice digits of a represent a * 2^q(S') to within 128/255 + 2^-8(S-S')
    # units (the dropped tail is a signed number below 0.502 units, the floor adds less than one unit of
    # the last of the S digits): what a tile with S' < S slices relies on
    rng = np.random.default_rng(S * 31 + Sp)
    n = S - Sp
    for _ in range(300):
        e_row = int(rng.integers(-40, 40))
        a = float(np.ldexp(rng.uniform(-1, 1), e_row - int(rng.integers(0, 60))))
        if abs(a) >= 2.0 ** (e_row + 1):
            continue
        d = oz.remap_unsigned_to_signed(oz.fixed_point(a, e_row, S), S)
        lead = sum(int(d[s]) * 256 ** (Sp - 1 - s) for s in range(Sp))
        want = Fraction(a) * Fraction(2) ** (8 * Sp - 2 - oz.H - e_row)
        assert abs(lead - want) <= Fraction(128, 255) + Fraction(1, 256 ** n)
        assert -128 <= d[0] <= 127 and abs(lead) <= 2 ** (8 * Sp - 2)      # still inside the headroom bit


def test_recompose_tiles_reduces_to_recompose():
    rng = np.random.default_rng(5)
    A, B = _structured(rng, 6, 40, 5, [2], 20)
    tr = oz.emulated_dgemm(A, B, mode=oz.MODE_FIXED_UNGUARDED, slices=9)
    full = oz.recompose(tr.P, tr.eA, tr.eB)
    np.testing.assert_array_equal(oz.recompose_tiles(tr.P, tr.eA, tr.eB, np.full((3, 3), 9), 2), full)
    # a tile with fewer slices equals the recomposition of the truncated planes on that tile only
    S_tile = np.full((3, 3), 9)
    S_tile[1, 2] = 7
    out = oz.recompose_tiles(tr.P, tr.eA, tr.eB, S_tile, 2)
    seven = oz.recompose(tr.P[:, :7], tr.eA, tr.eB)
    np.testing.assert_array_equal(out[2:4, 4:5], seven[2:4, 4:5])
    out[2:4, 4:5] = full[2:4, 4:5]
    np.testing.assert_array_equal(out, full)


@pytest.mark.parametrize("seed", range(16))
def test_per_tile_slice_counts_meet_the_bound(seed):
    # brute force against exact rationals: one wide row makes its tiles need more slices than the
    # rest; every tile, with its own slice count, stays inside k*2^-53 componentwise
    rng = np.random.default_rng(500 + seed)
    m, k, n, tile = 6, int(rng.integers(4, 24)), 6, 2
    spread = int(rng.integers(12, 45))
    A, B = _structured(rng, m, k, n, [int(rng.integers(m))], spread)
    b = int(rng.choice([1, 2, 8]))
    tr = oz.emulated_dgemm(A, B, mode=oz.MODE_DYNAMIC, max_bits=200, esc_block=b, per_tile=True, tile=tile)
    whole = oz.emulated_dgemm(A, B, mode=oz.MODE_DYNAMIC, max_bits=200, esc_block=b)
    assert tr.verdict.fallback == 0 and tr.verdict.slices_used == whole.verdict.slices_used
    assert tr.S_tile.max() == tr.verdict.slices_used and tr.S_tile.min() < tr.S_tile.max()
    np.testing.assert_array_equal(tr.S_tile, oz.tile_slices(53, oz.esc_coarse_tiles(A, B, b, tile)))
    fr = ex.exact_gemm_fraction(A, B)
    den = ex.bound_denominator(A, B)
    assert ex.gradeA_ratio(tr.C, fr, den, k) <= 1.0
    # tiles at the full count are untouched; the calm tiles really ran with fewer anti-diagonals
    full = tr.S_tile == tr.S_tile.max()
    for ti in range(3):
        for tj in range(3):
            r, c = slice(2 * ti, 2 * ti + 2), slice(2 * tj, 2 * tj + 2)
            if full[ti, tj]:
                np.testing.assert_array_equal(tr.C[r, c], whole.C[r, c])
    # negative control: one slice fewer than its ESC asks for breaks a wide tile's bound
    short = oz.recompose_tiles(tr.P, tr.eA, tr.eB, np.where(full, tr.S_tile - 3, tr.S_tile), tile)
    assert ex.gradeA_ratio(short, fr, den, k) > 1.0


def test_verdict_counts_pairs_per_tile():
    V = oz.verdict
    tile_esc = np.array([[1, 9], [17, 1]])
    v = V(oz.MODE_DYNAMIC, 53, 200, 0, False, 17, 512, 512, 64, None, tile_esc)
    assert (v.fallback, v.slices_used, v.slices_min, v.pair_tiles) == (0, 9, 7, 28 + 36 + 45 + 28)
    v = V(oz.MODE_DYNAMIC, 53, 200, 0, False, 17, 512, 512, 64)
    assert (v.slices_used, v.slices_min, v.pair_tiles) == (9, 9, 4 * 45)
    v = V(oz.MODE_FORCED_GUARDED, 53, 55, 0, False, 17, 300, 600, 64)
    assert (v.slices_used, v.slices_min, v.pair_tiles) == (7, 7, 2 * 3 * 28)
    assert V(oz.MODE_DYNAMIC, 53, 60, 0, False, 17, 512, 512, 64, None, tile_esc).reason == oz.REASON_BITS
    # the cost model sees the mean pair count: a single wide tile among many calm ones still pays
    hm = oz.HeuristicModel()
    n = 8192
    calm = np.ones((32, 32), dtype=np.int64)
    calm[3, 4] = 40                                            # S = 12 there, 7 elsewhere
    assert V(oz.MODE_DYNAMIC, 53, 200, 0, False, 40, n, n, n, hm).reason == oz.REASON_HEURISTIC
    v = V(oz.MODE_DYNAMIC, 53, 200, 0, False, 40, n, n, n, hm, calm)
    assert (v.fallback, v.slices_used, v.slices_min, v.pair_tiles) == (0, 12, 7, 1023 * 28 + 78)


# ---- the cost model of the run-time heuristic: invariants that any sign or term error breaks ----
def test_heuristic_closed_forms_and_monotonicity():
    # no fixed cost, free streaming: "slower" is exactly pairs / R_int8 > 1 / R_fp64
    hm = oz.HeuristicModel(int8_ops_per_ns=1000, fp64_flops_per_ns=40, bytes_per_ns=10 ** 12, fixed_ns=0)
    n = 4096
    for S in range(1, 27):
        assert hm.emulation_slower(S, n, n, n) == (oz.pairs_of(S) > 25)        # 1000 / 40
    # defaults: more slices never make emulation look faster; an explicit pair count overrides S's own
    hm = oz.HeuristicModel()
    for (m, n, k) in ((8192, 8192, 8192), (4096, 4096, 4096), (16384, 16384, 512), (256, 8192, 8192), (64, 64, 64)):
        seen = False
        for S in range(1, 27):
            slow = hm.emulation_slower(S, m, n, k)
            assert not (seen and not slow)
            seen = seen or slow
        assert hm.emulation_slower(7, m, n, k) == hm.emulation_slower(7, m, n, k, 28)
        assert hm.emulation_slower(7, m, n, k, 400)
    # cubes: one crossover size, small ones native (fixed cost and streaming dominate), large ones emulated
    slow = [hm.emulation_slower(7, n, n, n) for n in (32, 128, 512, 1024, 2048, 4096, 8192, 16384)]
    assert slow[0] and not slow[-1] and slow == sorted(slow, reverse=True)
    # the streaming term counts what the stages move: starving the bandwidth flips a winning case
    starved = oz.HeuristicModel(bytes_per_ns=50)
    assert not hm.emulation_slower(7, 8192, 8192, 8192) and starved.emulation_slower(7, 8192, 8192, 8192)
    # rational re-statement of the model at one point (integer floors only move it by < 3 ns)
    S, m, n, k = 8, 6000, 5000, 7000
    t_emu = Fraction(hm.fixed_ns) + Fraction(2 * m * n * k, hm.int8_ops_per_ns) * 36 + \
        Fraction((16 + S) * (m * k + k * n) + (2 * S + 22) * m * n, hm.bytes_per_ns)
    t_f64 = Fraction(2 * m * n * k, hm.fp64_flops_per_ns)
    assert abs(t_emu - t_f64) > 40                     # the decision is not a rounding accident
    assert hm.emulation_slower(S, m, n, k) == (t_emu > t_f64)


# ---- complex product by the 4M method ------------------------------------------------------------
def _cexact(A, B, alpha, beta, C):
    """Exact complex alpha*A*B + beta*C as pairs of Fractions."""
    F = lambda x: Fraction(float(x))
    m, k = A.shape
    n = B.shape[1]
    out = [[None] * n for _ in range(m)]
    ar, ai, br, bi = F(alpha.real), F(alpha.imag), F(beta.real), F(beta.imag)
    for i in range(m):
        for j in range(n):
            pr = sum((F(A[i, l].real) * F(B[l, j].real) - F(A[i, l].imag) * F(B[l, j].imag) for l in range(k)), Fraction(0))
            pi = sum((F(A[i, l].real) * F(B[l, j].imag) + F(A[i, l].imag) * F(B[l, j].real) for l in range(k)), Fraction(0))
            re, im = ar * pr - ai * pi, ar * pi + ai * pr
            if beta != 0:
                re += br * F(C[i, j].real) - bi * F(C[i, j].imag)
                im += br * F(C[i, j].imag) + bi * F(C[i, j].real)
            out[i][j] = (re, im)
    return out


@pytest.mark.parametrize("seed", range(6))
def test_zgemm_4m_meets_the_componentwise_bound(seed):
    # against exact rational arithmetic: real and imaginary part each within (k + 4) 2^-53 of
    # (|ar| + |ai|) (|Ar| + |Ai|)(|Br| + |Bi|) + (|br| + |bi|) (|Cr| + |Ci|), the bound the four
    # real products and the final combination add up to; a wrong sign or a swapped part breaks it
    rng = np.random.default_rng(700 + seed)
    m, k, n = int(rng.integers(1, 6)), int(rng.integers(1, 40)), int(rng.integers(1, 6))
    cplx = lambda shape: (rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * np.exp2(rng.integers(-6, 7, shape))
    A, B, C = cplx((m, k)), cplx((k, n)), cplx((m, n))
    alpha, beta = complex(1.25, -0.5), (complex(0.5, 2.0) if seed % 2 else 0.0)
    got, verdicts = oz.emulated_zgemm(A, B, alpha, beta, C, mode=oz.MODE_DYNAMIC, max_bits=200)
    assert len(verdicts) == 4 and all(v.fallback == 0 for v in verdicts)
    want = _cexact(A, B, complex(alpha), complex(beta), C)
    absA, absB = np.abs(A.real) + np.abs(A.imag), np.abs(B.real) + np.abs(B.imag)
    den = (abs(alpha.real) + abs(alpha.imag)) * (absA @ absB)
    if beta != 0:
        den = den + (abs(complex(beta).real) + abs(complex(beta).imag)) * (np.abs(C.real) + np.abs(C.imag))
    tol = (k + 4) * 2.0 ** -53
    worst = 0.0
    for i in range(m):
        for j in range(n):
            er = abs(Fraction(float(got[i, j].real)) - want[i][j][0])
            ei = abs(Fraction(float(got[i, j].imag)) - want[i][j][1])
            worst = max(worst, float(max(er, ei)) / (tol * den[i, j]))
    assert worst <= 1.0, worst
    # negative control: the conjugate product is far outside
    bad, _ = oz.emulated_zgemm(A, np.conj(B), alpha, beta, C, mode=oz.MODE_DYNAMIC, max_bits=200)
    if k > 2:
        assert np.max(np.abs(bad - got)) > 1e-6 * np.max(np.abs(got))


def test_zgemm_reduces_to_the_real_product():
    # purely real operands: the 4M product is the real emulated product, imaginary part exactly zero
    rng = np.random.default_rng(9)
    A, B = rng.standard_normal((5, 30)), rng.standard_normal((30, 4))
    got, verdicts = oz.emulated_zgemm(A + 0j, B + 0j, mode=oz.MODE_DYNAMIC, max_bits=200)
    real = oz.emulated_dgemm(A, B, mode=oz.MODE_DYNAMIC, max_bits=200)
    np.testing.assert_array_equal(got.real, real.C)
    assert np.all(got.imag == 0.0)
    assert verdicts[0] == real.verdict
    # i * (real product): multiplying A by i moves the product to the imaginary part, sign included
    got_i, _ = oz.emulated_zgemm(1j * A, B + 0j, mode=oz.MODE_DYNAMIC, max_bits=200)
    np.testing.assert_array_equal(got_i.imag, real.C)
    assert np.all(got_i.real == 0.0)
    # Inf/NaN in one part sends only the products that touch it to the native path
    A2 = A + 0j
    A2[1, 2] = complex(1.0, np.inf)
    _, v = oz.emulated_zgemm(A2, B + 1j * B, mode=oz.MODE_DYNAMIC, max_bits=200)
    assert [x.fallback for x in v] == [0, 1, 0, 1] and v[1].reason == oz.REASON_INFNAN
