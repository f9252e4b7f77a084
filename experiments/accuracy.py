#!/usr/bin/env python3
"""Accuracy experiments of the paper's section "Numerical Accuracy", run through the HIP library.

  test2   generalised BLAS-grading Test 2 (aspect A1): n = 1024, exponent-range parameter b swept,
          several mantissa-bit settings, without guardrails (FIXED_UNGUARDED) and with guardrails
          and automatic fallback (FIXED_GUARDED with target_bits = 53: the guard trips when
          53 + ESC exceeds the configured bits, so settings below 54 bits always fall back).  Error measure as in the paper: diagonal entries
          against x^T x accumulated in extended precision (FP80), off-diagonal entries against a
          reference O(n^3) floating-point product.
  gradeA  maximum and average componentwise relative error |fl(AB) - AB| / (|A||B|) against n for
          U(0,1) squares, five seeds (aspect A2): emulated (DYNAMIC, up to 200 bits), emulated
          forced to 55 bits, and the native FP64-MFMA kernel.  The "exact" product is the emulated
          product with 14 slices (>= 100 mantissa bits), itself checked on sampled entries against
          exact rational arithmetic (tests/test_gpu_parity.py::test_grade_a_sweep_uniform01 repeats the
          sweep at two sizes against the exact reference alone).

Writes plain-text tables next to this file (experiments/results/).  Inputs are the seeded generators
of paper_2511_13778_amd/workloads.py; nothing is read from outside the repository.
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "results")


def run(g, h, A, B, **opt):
    import torch
    m, k = A.shape
    n = B.shape[1]
    gm = g.Gemm(h, m, n, k, g.make_opts(**opt))
    dA, dB = g.to_colmajor(A), g.to_colmajor(B)
    dC = torch.empty((n, m), dtype=torch.float64, device="cuda")
    gm.run(dA, m, dB, k, dC, m)
    torch.cuda.synchronize()
    return g.from_colmajor(dC).copy(), gm.result()


def test2(g, h, nn, bits_list, b_list, seed, lines):
    from paper_2511_13778_amd import workloads as wl
    lines.append("# generalised Test 2, n = %d, seed %d: max relative error (diag vs FP80 x^T x, off-diag vs FP64 reference)" % (nn, seed))
    lines.append("# columns: b | ESC | per mantissa-bit setting: unguarded error, guarded error (F = fell back to native FP64)")
    lines.append("b    ESC  " + "  ".join("%3d-bit:unguarded  guarded " % mb for mb in bits_list))
    for b in b_list:
        A, B, x = wl.grading_test2(nn, b, seed)
        xl = x.astype(np.longdouble)
        diag = float(np.sum(xl * xl))
        with np.errstate(all="ignore"):
            ref = A @ B
        off = ~np.eye(nn, dtype=bool)

        def err(C):
            with np.errstate(all="ignore"):
                e_diag = np.max(np.abs(np.diag(C) - diag) / diag)
                e_off = np.max(np.abs(C[off] - ref[off]) / np.abs(ref[off]))
            return float(max(e_diag, e_off))
        row, esc = [], None
        for mb in bits_list:
            Cu, _ = run(g, h, A, B, mode=g.OZ_FIXED_UNGUARDED, max_bits=mb, heuristic=0)
            Cg, rg = run(g, h, A, B, mode=g.OZ_FIXED_GUARDED, target_bits=53, max_bits=mb, heuristic=0)
            esc = rg.esc
            row.append("%18.3e  %8.2e%s" % (err(Cu), err(Cg), "F" if rg.fallback else " "))
        lines.append("%-4d %-4d " % (b, esc) + "  ".join(row))


def grade_a(g, h, sizes, seeds, lines):
    from fractions import Fraction
    from paper_2511_13778_amd import workloads as wl

    def exact_entry(A, B, i, j):
        """(A B)_ij in exact rational arithmetic, rounded once: pins the many-slice reference on sampled entries"""
        return float(sum((Fraction(float(a)) * Fraction(float(b)) for a, b in zip(A[i, :], B[:, j])), Fraction(0)))

    eps = 2.0 ** -53
    lines.append("# componentwise relative error |fl(AB)-AB| / (|A||B|) in units of eps = 2^-53; U(0,1) squares; %d seeds" % len(seeds))
    lines.append("# grade A requires max error <= f(n)*eps with f at most linear in n; the last column is n (the allowed slope)")
    lines.append("n      | emulated dynamic: max avg slices | emulated 55-bit: max avg | native FP64 MFMA: max avg | n")
    for nn in sizes:
        acc = {"dyn": [], "f55": [], "nat": []}
        slices = set()
        for seed in seeds:
            A, B = wl.uniform_01(nn, nn, nn, seed)
            den = np.abs(A) @ np.abs(B)
            ref, rr = run(g, h, A, B, mode=g.OZ_FIXED_UNGUARDED, slices=14, heuristic=0)
            idx = [(int(i), int(j)) for i, j in np.random.default_rng(seed).integers(0, nn, (24, 2))]
            exact = [exact_entry(A, B, i, j) for i, j in idx]
            assert max(abs(ref[i, j] - e) for (i, j), e in zip(idx, exact)) <= 2 * eps * float(den.max()), "reference product is off"
            for key, opt in (("dyn", dict(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0)),
                             ("f55", dict(mode=g.OZ_FORCED_GUARDED, max_bits=55, heuristic=0)),
                             ("nat", dict(mode=g.OZ_NATIVE))):
                C, res = run(g, h, A, B, **opt)
                e = np.abs(C - ref) / den / eps
                acc[key].append((float(e.max()), float(e.mean())))
                if key == "dyn":
                    assert res.fallback == 0, "dynamic mode fell back"
                    slices.add(res.slices_used)
        fmt = lambda v: "%8.3f %8.4f" % (max(t[0] for t in v), float(np.mean([t[1] for t in v])))
        lines.append("%-6d | %s %s | %s | %s | %d" % (nn, fmt(acc["dyn"]), sorted(slices), fmt(acc["f55"]), fmt(acc["nat"]), nn))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["test2", "gradeA", "all"])
    ap.add_argument("--n", type=int, default=1024)
    ap.add_argument("--sizes", default="256,512,1024,2048,4096")
    ap.add_argument("--seeds", type=int, default=5)
    args = ap.parse_args()
    from paper_2511_13778_amd import ozdgemm as g
    h = g.Handle(0)
    os.makedirs(OUT, exist_ok=True)
    if args.what in ("test2", "all"):
        lines = []
        test2(g, h, args.n, [31, 39, 47, 55, 63, 79], [0, 5, 10, 15, 20, 25, 30, 40, 60, 100, 200, 400], 1, lines)
        open(os.path.join(OUT, "test2_n%d.txt" % args.n), "w").write("\n".join(lines) + "\n")
        print("\n".join(lines))
    if args.what in ("gradeA", "all"):
        lines = []
        grade_a(g, h, [int(v) for v in args.sizes.split(",")], list(range(1, args.seeds + 1)), lines)
        open(os.path.join(OUT, "gradeA_uniform01.txt"), "w").write("\n".join(lines) + "\n")
        print("\n".join(lines))
    h.close()


if __name__ == "__main__":
    main()
