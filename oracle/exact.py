"""Exact reference for C = alpha*A*B + beta*C and the componentwise error measure.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT (see oracle/ozaki.py).  Two independent routes:
  * exact_gemm_fraction: rational arithmetic, tiny inputs;
  * exact_dot_fsum / exact_entries: every product a*b is split without error into a rounded
    product and its rounding error (Veltkamp/Dekker splitting, valid while nothing over- or
    underflows), and math.fsum, which returns the correctly rounded sum of its arguments,
    adds all 2k pieces.  The result is the exact dot product rounded once to FP64.
The acceptance measure is the componentwise (Grade A) bound of section "Numerical Accuracy",
aspect A2:  |C - C_exact|_ij <= f * eps * (|alpha| |A||B| + |beta| |C_in|)_ij  with f*eps = k*2^-53.
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np


def exact_gemm_fraction(A, B, alpha=1.0, beta=0.0, C=None):
    """m x n list of Fractions: alpha*A*B + beta*C exactly."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    m, k = A.shape
    n = B.shape[1]
    FA = [[Fraction(float(A[i, l])) for l in range(k)] for i in range(m)]
    FB = [[Fraction(float(B[l, j])) for j in range(n)] for l in range(k)]
    fa, fb = Fraction(float(alpha)), Fraction(float(beta))
    out = [[None] * n for _ in range(m)]
    for i in range(m):
        for j in range(n):
            s = sum((FA[i][l] * FB[l][j] for l in range(k)), Fraction(0))
            s = fa * s
            if beta != 0.0:
                s += fb * Fraction(float(C[i, j]))
            out[i][j] = s
    return out


_SPLIT = 134217729.0  # 2^27 + 1


def _two_product(a: np.ndarray, b: np.ndarray):
    """p = fl(a*b) and e with a*b = p + e exactly (Dekker), elementwise."""
    p = a * b
    ca = _SPLIT * a
    ah = ca - (ca - a)
    al = a - ah
    cb = _SPLIT * b
    bh = cb - (cb - b)
    bl = b - bh
    e = ((ah * bh - p) + ah * bl + al * bh) + al * bl
    return p, e


def exact_dot_fsum(x: np.ndarray, y: np.ndarray, extra=()) -> float:
    """Correctly rounded value of sum_l x_l*y_l + sum(extra products), extra = [(u, v), ...]."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    p, e = _two_product(x, y)
    terms = list(p) + list(e)
    for u, v in extra:
        pu, eu = _two_product(np.float64(u), np.float64(v))
        terms += [float(pu), float(eu)]
    return math.fsum(terms)


def _int_parts(v: np.ndarray):
    """v = M * 2^e elementwise with M an integer of at most 53 bits (object array) and e int."""
    f, p = np.frexp(np.asarray(v, dtype=np.float64))
    M = (f * 9007199254740992.0).astype(np.int64).astype(object)     # f * 2^53 is an exact integer
    return M, p.astype(np.int64) - 53


def exact_dot_fraction(x: np.ndarray, y: np.ndarray) -> Fraction:
    """sum_l x_l*y_l as an exact rational, accumulated in Python integers:
    each product is Mx*My * 2^(ex+ey); all are shifted to the smallest exponent and added."""
    Mx, ex = _int_parts(x)
    My, ey = _int_parts(y)
    e = ex + ey
    emin = int(e.min()) if len(e) else 0
    total = int(np.sum((Mx * My) * (2 ** (e - emin).astype(object)), initial=0))
    return Fraction(total) * Fraction(2) ** emin


def exact_entries(A, B, idx, alpha=1.0, beta=0.0, C=None):
    """Correctly rounded alpha*(A*B)_ij + beta*C_ij for the sampled (i, j) in idx.

    alpha == 1: every term is an error-free product, added by fsum.  Otherwise the dot product
    is accumulated exactly in integers, combined with alpha and beta*C as rationals, and rounded
    once by the conversion to float."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    out = np.empty(len(idx), dtype=np.float64)
    fa, fb = Fraction(float(alpha)), Fraction(float(beta))
    for t, (i, j) in enumerate(idx):
        if alpha == 1.0:
            extra = [(beta, C[i, j])] if beta != 0.0 else []
            out[t] = exact_dot_fsum(A[i, :], B[:, j], extra)
        else:
            s = fa * exact_dot_fraction(A[i, :], B[:, j])
            if beta != 0.0:
                s += fb * Fraction(float(C[i, j]))
            out[t] = float(s)          # Fraction -> float rounds correctly
    return out


def bound_denominator(A, B, idx=None, alpha=1.0, beta=0.0, C=None):
    """(|alpha| |A||B| + |beta| |C_in|)_ij, in FP64 (its own rounding is irrelevant at 2^-53)."""
    A = np.abs(np.asarray(A, dtype=np.float64))
    B = np.abs(np.asarray(B, dtype=np.float64))
    if idx is None:
        den = abs(alpha) * (A @ B)
        if beta != 0.0:
            den = den + abs(beta) * np.abs(C)
        return den
    den = np.array([abs(alpha) * float(A[i, :] @ B[:, j]) for i, j in idx])
    if beta != 0.0:
        den = den + abs(beta) * np.array([abs(C[i, j]) for i, j in idx])
    return den


def gradeA_ratio(C_got, C_exact, den, k: int) -> float:
    """max_ij |C_got - C_exact| / (den * k * 2^-53); <= 1 means the bound holds.
    Entries whose denominator is 0 must match exactly (ratio inf otherwise)."""
    got = np.asarray(C_got, dtype=np.float64).ravel()
    if isinstance(C_exact, list):
        ex = [x for row in C_exact for x in row]
        err = np.array([float(abs(Fraction(float(g)) - e)) for g, e in zip(got, ex)])
    else:
        err = np.abs(got - np.asarray(C_exact, dtype=np.float64).ravel())
    den = np.asarray(den, dtype=np.float64).ravel() * (k * 2.0 ** -53)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.where(den > 0, err / den, np.where(err == 0, 0.0, np.inf))
    return float(r.max(initial=0.0))
