"""Pins for the oracle's slicing (O5): the paper's printed example, exact reconstruction of
floor(a*2^q), range of the digits, agreement of the vectorised and the big-integer routes."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ozaki as oz

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_printed_example():
    hi_u, lo_u, hi_s, lo_s, pattern = _rows("unsigned_slice_example.txt")[0]
    X = int(hi_u) * 256 + int(lo_u)
    assert oz.remap_unsigned_to_signed(X, 2) == [int(hi_s), int(lo_s)]
    assert int(lo_s) & 0xFF == int(pattern, 2) == int(lo_u)


def test_slice_counts_from_paper():
    bits, s_signed, s_unsigned, pct = map(int, _rows("slice_counts.txt")[0])
    assert oz.slices_signed_scheme(bits) == s_signed
    assert oz.slices_for_bits(bits) == s_unsigned
    assert oz.slices_for_bits(55) == s_unsigned
    p7 = sum(len(d) for d in oz.kept_pairs(s_unsigned))
    p8 = sum(len(d) for d in oz.kept_pairs(s_signed))
    assert (p7, p8) == (28, 36)
    assert round(100 * (1 - p7 / p8)) == pct          # 22 %; full squares 49/64 would give 23
    assert round(100 * (1 - 49 / 64)) != pct


def test_remap_exhaustive_two_and_three_bytes():
    for S, lim in ((2, 1 << 14), (3, 1 << 15)):
        for X in range(-lim, lim, 1 if S == 2 else 7):
            d = oz.remap_unsigned_to_signed(X, S)
            assert all(-128 <= v <= 127 for v in d)
            assert sum(v * 256 ** (S - 1 - s) for s, v in enumerate(d)) == X
            # bytes of the digits are the bytes of X + 0x..8080 with the top bit of every
            # sub-leading byte flipped: the "same bit pattern" property of the encoding
            Y = X + sum(128 * 256 ** (S - 1 - s) for s in range(1, S))
            for s in range(1, S):
                assert (d[s] & 0xFF) == ((Y >> (8 * (S - 1 - s))) & 0xFF) ^ 0x80


def test_headroom_bit_is_needed():
    # without headroom the carry can push the leading digit to 128
    with pytest.raises(AssertionError):
        oz.remap_unsigned_to_signed(0x7F80, 2)
    # with |X| < 2^(8S-2) it cannot
    assert oz.remap_unsigned_to_signed(0x3FFF, 2) == [64, -1]


def _edge_values():
    tiny = 5e-324
    return np.array([1.0, -1.0, 1.5, -1.5, 2.0 - 2.0 ** -52, -(2.0 - 2.0 ** -52), 0.0, -0.0,
                     1.0 + 2.0 ** -52, 0.75, -0.3, 1e-3, -1e-5, 2.0 ** -40, -(2.0 ** -60),
                     tiny, -tiny, 2.2250738585072014e-308, 1.1e-308, -3.3e-310,
                     123456789.123, -0.999999999999, 2.0 ** -1074 * 12345], dtype=np.float64)


@pytest.mark.parametrize("S", [1, 2, 5, 7, 8, 9, 12, 26])
def test_digits_reconstruct_floor(S):
    rng = np.random.default_rng(100 + S)
    v = np.concatenate([_edge_values(), rng.standard_normal(40) * np.exp(3 * rng.standard_normal(40))])
    for scale_e in (0, -1000, 900):
        w = np.ldexp(v, scale_e) if scale_e else v
        w = w[np.isfinite(w)]
        e_row = int(oz.exponents(w).max())
        D = oz.slice_vector_exact(w, e_row, S).astype(np.int64)
        q = 8 * S - 3 - e_row
        for l, a in enumerate(w):
            X = sum(int(D[s, l]) * 256 ** (S - 1 - s) for s in range(S))
            assert X == math.floor(Fraction(float(a)) * Fraction(2) ** q)
            assert abs(X) < 1 << (8 * S - 2) or X == -(1 << (8 * S - 2))
            assert -64 <= D[0, l] <= 64


def test_enough_slices_are_exact():
    # entries within 2^-10 of the row maximum: 8S-2 >= 53+10 makes a*2^q an integer
    rng = np.random.default_rng(5)
    v = rng.uniform(1.0, 2.0, 50) * np.ldexp(1.0, -rng.integers(0, 11, 50))
    e_row = int(oz.exponents(v).max())
    S = 9
    D = oz.slice_vector_exact(v, e_row, S).astype(np.int64)
    for l, a in enumerate(v):
        X = sum(int(D[s, l]) * 256 ** (S - 1 - s) for s in range(S))
        assert Fraction(X) == Fraction(float(a)) * Fraction(2) ** (8 * S - 3 - e_row)


@pytest.mark.parametrize("S", [1, 7, 9, 26])
def test_shift_route_matches_rationals(S):
    rng = np.random.default_rng(70 + S)
    v = np.concatenate([_edge_values(), rng.standard_normal(60) * np.exp2(rng.integers(-80, 80, 60))])
    for e_extra in (0, 5, 300):
        e_row = int(oz.exponents(v).max()) + e_extra
        for a in v:
            assert oz.fixed_point_shift(float(a), e_row, S) == oz.fixed_point(float(a), e_row, S)
    A = v[:24].reshape(4, 6)
    eA = oz.row_exponents(A)
    np.testing.assert_array_equal(oz.slice_rows_bigint(A, eA, S), oz.slice_rows_exact(A, eA, S))


@pytest.mark.parametrize("S", [1, 3, 7, 8])
def test_vectorised_route_matches_big_integers(S):
    rng = np.random.default_rng(7 + S)
    A = rng.standard_normal((9, 31)) * np.exp(4 * rng.standard_normal((9, 31)))
    A[0, :len(_edge_values())] = _edge_values()
    A[1, :] = 0.0
    A[2, 3] = 0.0
    A[3, :] = np.ldexp(rng.uniform(-1, 1, 31), -1060)      # denormal row
    A[4, :] = -(2.0 - 2.0 ** -52)
    eA = oz.row_exponents(A)
    assert eA[1] == oz.ZERO_EXP
    np.testing.assert_array_equal(oz.slice_rows_int64(A, eA, S), oz.slice_rows_exact(A, eA, S))


def test_power_of_two_row_scaling_leaves_digits_unchanged():
    rng = np.random.default_rng(11)
    A = rng.uniform(-1, 1, (6, 40))
    scaled = A * np.ldexp(1.0, np.arange(6) * 7 - 20)[:, None]
    d0 = oz.slice_rows(A, oz.row_exponents(A), 7)
    d1 = oz.slice_rows(scaled, oz.row_exponents(scaled), 7)
    np.testing.assert_array_equal(d0, d1)
