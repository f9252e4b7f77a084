#!/usr/bin/env python3
"""Blocked Householder QR with its trailing-matrix update through oz_dgemm (the paper's section
"Application-Level Integration"): run time against the same driver with the native FP64 GEMM, and the
distribution of slice counts / fallbacks the decision process chose over one factorisation.

For each size and panel width:
  native            every trailing-update GEMM on this library's FP64-MFMA kernel (OZ_NATIVE)
  shipped           oz_default_opts: OZ_DYNAMIC, run-time heuristic on, per-block slice counts
  dynamic           OZ_DYNAMIC with the heuristic off: everything emulated, slice counts from the ESC
  fixed 55          OZ_FIXED_UNGUARDED with 7 slices: the paper's "upper bound" configuration
plus torch.geqrf on the whole matrix (the vendor solver) for scale.  Accuracy: ||A^T A - R^T R||_F /
||A||_F^2 (independent of Q) in units of n * 2^-53.

Writes experiments/results/qr.txt.  Inputs: i.i.d. N(0,1) from a seeded generator on the device.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "results")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sizes", default="8192")
    ap.add_argument("--panels", default="256,1024")
    ap.add_argument("--out", default=os.path.join(OUT, "qr.txt"))
    args = ap.parse_args()
    import torch
    from paper_2511_13778_amd import ozdgemm as g
    from paper_2511_13778_amd.qr import blocked_qr

    h = g.Handle(0)
    configs = [("native", g.make_opts(mode=g.OZ_NATIVE)),
               ("shipped", g.default_opts()),
               ("dynamic", g.make_opts(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0, tile_slices=1)),
               ("fixed 55", g.make_opts(mode=g.OZ_FIXED_UNGUARDED, max_bits=55))]
    lines = ["# blocked Householder QR, trailing update through oz_dgemm; total = whole factorisation (panel factorisation",
             "# by torch.geqrf included), gemm = the trailing-update products alone (HIP events), both in ms, best of 2;",
             "# x native = native gemm time / this gemm time; residual = ||A^T A - R^T R||_F / ||A||_F^2 in units of 2^-53",
             "# histogram: GEMM calls of one factorisation by outcome (S = slice count of an emulated call)"]
    for n in [int(v) for v in args.sizes.split(",")]:
        gen = torch.Generator(device="cuda").manual_seed(1234 + n)
        A0t = torch.randn((n, n), dtype=torch.float64, device="cuda", generator=gen)     # column-major A
        AtA = A0t @ A0t.T
        nrm2 = float(torch.linalg.matrix_norm(A0t) ** 2)
        torch.geqrf(A0t.T.contiguous())
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        torch.geqrf(A0t.T.contiguous())
        torch.cuda.synchronize()
        t_vendor = (time.perf_counter() - t0) * 1e3
        lines.append("")
        lines.append("## n = %d   (torch.geqrf on the whole matrix: %.1f ms)" % (n, t_vendor))
        lines.append("panel  mode      total     gemm      x native  residual  histogram")
        for b in [int(v) for v in args.panels.split(",")]:
            t_native = None
            for name, opts in configs:
                best = best_gemm = None
                for rep in range(2):
                    At = A0t.clone()
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    _, rep_ = blocked_qr(h, At, b, opts)
                    torch.cuda.synchronize()
                    dt = (time.perf_counter() - t0) * 1e3
                    best = dt if best is None else min(best, dt)
                    best_gemm = rep_.gemm_ms if best_gemm is None else min(best_gemm, rep_.gemm_ms)
                R = torch.triu(At.T)
                resid = float(torch.linalg.matrix_norm(AtA - R.T @ R)) / nrm2 / 2.0 ** -53
                if name == "native":
                    t_native = best_gemm
                hist = ", ".join("%s: %d" % kv for kv in sorted(rep_.histogram().items()))
                lines.append("%-6d %-9s %-9.1f %-9.1f %-9.2f %-9.3g %s" % (b, name, best, best_gemm, t_native / best_gemm, resid, hist))
                print(lines[-1], flush=True)
    os.makedirs(OUT, exist_ok=True)
    with open(args.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    h.close()


if __name__ == "__main__":
    main()
