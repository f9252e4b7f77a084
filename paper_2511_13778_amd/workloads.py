"""Seeded synthetic inputs shaped like the paper's workloads.

Holds no arithmetic of the method: only random matrices.  Both the CPU oracle's tests and the
HIP path's tests/benchmarks draw their inputs here, so they see identical data.  All matrices
are returned as C-contiguous numpy float64 arrays in logical (row, column) indexing; callers
choose the memory layout they hand to the library.

Recipes (performance inputs in the paper are unspecified "random matrices"; its accuracy
inputs are U(0,1) squares and the generalised Test-2 family of section "Numerical Accuracy"):
  uniform_pm1          i.i.d. U[-1,1]
  uniform_01           i.i.d. U(0,1)                       (aspect A2)
  lognormal_spread     (U(0,1)-0.5) * exp(phi*N(0,1))       (moderate/large exponent spread)
  row_scaled           U[-1,1], row i of A times 2^(i mod 40)
  wide_span            N(0,1) times 2^-300 or 2^+300, chosen per entry
  rank1_cancel         A = u v^T + 1e-12*N(0,1)
  grading_test2             A_{k,:} = x^T D P_k,  B_{:,k} = P_k^-1 D^-1 x,  x~U(1,2), D = diag(2^j)
  wide_rows            +-U(1,2) everywhere, except a band of rows of A whose dot products with every
                       third column of B have a large exponent span (a localised hard region)
"""
from __future__ import annotations

import numpy as np


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def uniform_pm1(m, k, n, seed):
    r = _rng(seed)
    return r.uniform(-1.0, 1.0, (m, k)), r.uniform(-1.0, 1.0, (k, n))


def uniform_01(m, k, n, seed):
    r = _rng(seed)
    return r.uniform(0.0, 1.0, (m, k)), r.uniform(0.0, 1.0, (k, n))


def lognormal_spread(m, k, n, phi, seed, with_c=False):
    r = _rng(seed)
    A = (r.uniform(0.0, 1.0, (m, k)) - 0.5) * np.exp(phi * r.standard_normal((m, k)))
    B = (r.uniform(0.0, 1.0, (k, n)) - 0.5) * np.exp(phi * r.standard_normal((k, n)))
    if with_c:
        return A, B, r.standard_normal((m, n))
    return A, B


def row_scaled(m, k, n, seed, period=40):
    r = _rng(seed)
    A0 = r.uniform(-1.0, 1.0, (m, k))
    B = r.uniform(-1.0, 1.0, (k, n))
    scale = np.ldexp(1.0, (np.arange(m) % period).astype(np.int32))
    return A0 * scale[:, None], B, A0


def wide_span(m, k, n, seed, lo=-300, hi=300):
    r = _rng(seed)
    def one(shape):
        e = np.where(r.integers(0, 2, shape) == 0, lo, hi).astype(np.int32)
        return np.ldexp(r.standard_normal(shape), e)
    return one((m, k)), one((k, n))


def plant_inf_nan(A, B, seed):
    """Copies of A, B with +Inf, -Inf and NaN written at three random places."""
    r = _rng(seed)
    A, B = A.copy(), B.copy()
    A[r.integers(A.shape[0]), r.integers(A.shape[1])] = np.inf
    B[r.integers(B.shape[0]), r.integers(B.shape[1])] = -np.inf
    A[r.integers(A.shape[0]), r.integers(A.shape[1])] = np.nan
    return A, B


def rank1_cancel(m, k, n, seed, noise=1e-12):
    r = _rng(seed)
    u, v = r.standard_normal(m), r.standard_normal(k)
    A = np.outer(u, v) + noise * r.standard_normal((m, k))
    B = r.standard_normal((k, n))
    return A, B


def grading_test2(nn, b, seed):
    """Generalised Test 2: exponent range parameter b (section "Numerical Accuracy", aspect A1).
    Returns A, B and x; the exact diagonal of A*B is x^T x."""
    r = _rng(seed)
    x = r.uniform(1.0, 2.0, nn)
    delta = 2.0 * b / (nn - 1) if nn > 1 else 0.0
    j = (-b + np.round(np.arange(nn) * delta)).astype(np.int32)
    xd = np.ldexp(x, j)
    xinv = np.ldexp(x, -j)
    A = np.empty((nn, nn))
    B = np.empty((nn, nn))
    for kk in range(nn):
        A[kk, :] = np.roll(xd, kk)
        B[:, kk] = np.roll(xinv, kk)
    return A, B, x


def wide_rows(m, k, n, seed, row_lo, row_hi, spread):
    """+-U(1,2) matrices (all exponents 0) with a band of difficult rows: each row i in [row_lo, row_hi)
    of A keeps one entry, at a random position l0, and is scaled by 2^-spread elsewhere; B[l0, j] is
    scaled by 2^-spread for every third column j.  The dot products (i, j) of the band with those
    columns then have no product within `spread` bits of the row and column maxima, all others do:
    only the blocks of C that meet the band need many mantissa bits."""
    r = _rng(seed)
    A = r.uniform(1.0, 2.0, (m, k)) * r.choice([-1.0, 1.0], (m, k))
    B = r.uniform(1.0, 2.0, (k, n)) * r.choice([-1.0, 1.0], (k, n))
    for i in range(row_lo, row_hi):
        l0 = int(r.integers(k))
        keep = A[i, l0]
        A[i] = np.ldexp(A[i], -spread)
        A[i, l0] = keep
        B[l0, ::3] = np.ldexp(B[l0, ::3], -spread)
    return A, B
