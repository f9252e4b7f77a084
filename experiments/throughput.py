#!/usr/bin/env python3
"""Throughput experiments of the paper's section "Performance", run through the HIP library.

For square sizes (default 8192; add 16384 with --sizes) and entries (U(0,1)-0.5)*exp(phi*N(0,1)),
phi in {0.1, 1, 2}, alpha = 1.5, beta = 0.5, random C:

  modes   effective FP64 TFLOP/s (2mnk/t) without guardrails at 55 bits (the ceiling), with
          guardrails forced to 55 bits (the paper's headline setting), in dynamic mode (slice count
          from the ESC), and of the two native FP64 GEMMs (this library's MFMA kernel, the vendor
          library through torch.matmul); share of the run time spent in the guardrails.
  slices  fixed slice count swept S = 4..12 without guardrails: time against S(S+1)/2.
  block   block length b of the coarsened ESC swept: reported ESC, slice count a dynamic run would
          take, and the time of the ESC stage.
  shapes  (--shapes) rectangular problems: the tall-skinny / long-k / short-k shapes with row i of
          A scaled by 2^(i mod 40), and the two GEMM shapes of a blocked QR trailing update;
          emulated (forced 55 bits) against both native FP64 GEMMs, and what the heuristic decides.

Writes plain-text tables next to this file (experiments/results/).  Inputs are the seeded
generators of paper_2511_13778_amd/workloads.py; nothing is read from outside the repository.
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "results")
ALPHA, BETA = 1.5, 0.5


def timed(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def emulated(torch, g, h, n, dA, dB, dC, reps, **opt):
    """ms per call, result record and mean stage times of one configuration"""
    gm = g.Gemm(h, n, n, n, g.make_opts(heuristic=0, **opt))
    fn = lambda: gm.run(dA, n, dB, n, dC, n, ALPHA, BETA)
    fn()
    torch.cuda.synchronize()
    h.profile_enable(reps)
    ms = timed(torch, fn, reps)
    # the first `reps` calls after profile_enable are recorded (timed() starts with one untimed call)
    stages = np.array([h.profile_read(c) for c in range(reps)]).mean(axis=0)
    res = gm.result()
    del gm
    return ms, res, dict(zip(g.STAGE_NAMES, stages))


SHAPES = [(16384, 16384, 512), (1024, 1024, 65536), (32768, 256, 8192), (4096, 4096, 4096), (2048, 2048, 2048),
          (256, 8192, 8192), (8192, 8192, 256)]


def shapes(torch, g, h, reps):
    from paper_2511_13778_amd import workloads as wl
    st = torch.cuda.current_stream().cuda_stream
    lines = ["# rectangular problems, row i of A scaled by 2^(i mod 40), alpha = 1, beta = 0; %d timed calls per entry" % reps,
             "# heuristic: what the library decides for this input with its default options (DYNAMIC, cost model on)",
             "# as shipped: that same call timed (scan, ESC and verdict included; its native GEMM may split k, using the workspace)",
             "m      n      k      | emulated forced 55: ms TFLOP/s (gemm recompose slicing ms) | own FP64 ms | vendor FP64 ms | x vendor | heuristic | as shipped ms"]
    for m, n, k in SHAPES:
        print("shape %d %d %d" % (m, n, k), flush=True)
        A, B, _ = wl.row_scaled(m, k, n, seed=6)
        dA, dB = g.to_colmajor(A), g.to_colmajor(B)
        del A, B
        dC = torch.zeros((n, m), dtype=torch.float64, device="cuda")
        gm = g.Gemm(h, m, n, k, g.make_opts(mode=g.OZ_FORCED_GUARDED, max_bits=55, heuristic=0))
        fn = lambda: gm.run(dA, m, dB, k, dC, m, 1.0, 0.0)
        fn()
        torch.cuda.synchronize()
        h.profile_enable(reps)
        ms = timed(torch, fn, reps)
        sm = dict(zip(g.STAGE_NAMES, np.array([h.profile_read(c) for c in range(reps)]).mean(axis=0)))
        t_own = timed(torch, lambda: h.native_dgemm(st, "N", "N", m, n, k, 1.0, dA.data_ptr(), m, dB.data_ptr(), k, 0.0,
                                                    dC.data_ptr(), m), reps)
        t_ven = timed(torch, lambda: torch.matmul(dB, dA), reps)
        gd = g.Gemm(h, m, n, k, g.default_opts())
        gd.run(dA, m, dB, k, dC, m, 1.0, 0.0)
        torch.cuda.synchronize()
        rd = gd.result()
        slower = bool(rd.fallback)
        t_ship = timed(torch, lambda: gd.run(dA, m, dB, k, dC, m, 1.0, 0.0), reps)
        del gd
        lines.append("%-6d %-6d %-6d | %8.3f %6.1f (%.3f %.3f %.3f) | %8.3f | %8.3f | %5.2f | %s | %.3f"
                     % (m, n, k, ms, 2.0 * m * n * k / ms * 1e-9, sm["slice_gemm_i8"], sm["recompose"], sm["slicing"],
                        t_own, t_ven, t_ven / ms, ("native (reason %d)" % rd.reason) if slower else "emulate, S = %d" % rd.slices_used,
                        t_ship))
        del dA, dB, dC, gm
        torch.cuda.empty_cache()
    with open(os.path.join(OUT, "throughput_shapes.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines), flush=True)


def localised(torch, g, h, reps):
    """A localised hard region: 100 rows of A whose dot products need many more bits than the rest
    (workloads.wide_rows).  One slice count for all of C against per-block counts, both against FP64."""
    from paper_2511_13778_amd import workloads as wl
    st = torch.cuda.current_stream().cuda_stream
    n = 8192
    lines = ["# m = n = k = %d, +-U(1,2) entries, rows 3000..3099 of A with a %%d-bit exponent span against every third column;"
             " alpha = 1, beta = 0; %d timed calls per entry" % (n, reps),
             "# 'cols': the transposed product, i.e. the hard region is a band of columns of C",
             "spread | mode                      S_max S_min pair products of 256x256 blocks   ms      TFLOP/s  x vendor FP64 x own FP64"]
    # the last case transposes the product (A <- B^T, B <- A^T): the same hard region as a band of columns of C
    for spread, columns in ((24, False), (40, False), (60, False), (24, True)):
        A, B = wl.wide_rows(n, n, n, seed=11, row_lo=3000, row_hi=3100, spread=spread)
        if columns:
            A, B = np.ascontiguousarray(B.T), np.ascontiguousarray(A.T)
        dA, dB = g.to_colmajor(A), g.to_colmajor(B)
        del A, B
        dC = torch.zeros((n, n), dtype=torch.float64, device="cuda")
        t_ven = timed(torch, lambda: torch.matmul(dB, dA), 3)
        t_own = timed(torch, lambda: h.native_dgemm(st, "N", "N", n, n, n, 1.0, dA.data_ptr(), n, dB.data_ptr(), n, 0.0,
                                                    dC.data_ptr(), n), 3)
        for name, opt in (("dynamic, one count", dict(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0, tile_slices=0)),
                          ("dynamic, per-block counts", dict(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0, tile_slices=1)),
                          ("as shipped (heuristic on)", None)):
            gm = g.Gemm(h, n, n, n, g.default_opts() if opt is None else g.make_opts(**opt))
            fn = lambda: gm.run(dA, n, dB, n, dC, n, 1.0, 0.0)
            ms = timed(torch, fn, reps)
            r = gm.result()
            what = "native (reason %d)" % r.reason if r.fallback else "%-5d %-5d %d" % (r.slices_used, r.slices_min, r.pair_tiles)
            lines[0] = lines[0]
            lines.append("%-6s | %-25s %-40s %-7.2f %-8.1f %-13.2f %.2f" % (("%d cols" % spread) if columns else str(spread), name, what, ms,
                                                                          2.0 * n ** 3 / ms * 1e-9, t_ven / ms, t_own / ms))
            del gm
        del dA, dB, dC
        torch.cuda.empty_cache()
    lines[0] = lines[0].replace("%d-bit", "given-bit")
    with open(os.path.join(OUT, "throughput_localised.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shapes", action="store_true")
    ap.add_argument("--localised", action="store_true")
    ap.add_argument("--sizes", default="8192")
    ap.add_argument("--phis", default="0.1,1,2")
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args()
    import torch
    from paper_2511_13778_amd import ozdgemm as g
    from paper_2511_13778_amd import workloads as wl
    if not torch.cuda.is_available():
        sys.exit("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
    os.makedirs(OUT, exist_ok=True)
    h = g.Handle(0)
    st = torch.cuda.current_stream().cuda_stream
    if args.shapes:
        shapes(torch, g, h, args.reps)
        h.close()
        return
    if args.localised:
        localised(torch, g, h, args.reps)
        h.close()
        return
    for n in (int(v) for v in args.sizes.split(",")):
        flops = 2.0 * n ** 3
        tf = lambda ms: flops / (ms * 1e-3) * 1e-12
        lines = ["# m = n = k = %d, alpha = %g, beta = %g, %d timed calls per entry; TFLOP/s = 2mnk/t" % (n, ALPHA, BETA, args.reps)]
        for phi in (float(v) for v in args.phis.split(",")):
            print("size %d phi %g: generating" % (n, phi), flush=True)
            A, B, Cin = wl.lognormal_spread(n, n, n, phi, seed=4, with_c=True)
            dA, dB, dC = g.to_colmajor(A), g.to_colmajor(B), g.to_colmajor(Cin)
            del A, B, Cin
            t_own = timed(torch, lambda: h.native_dgemm(st, "N", "N", n, n, n, ALPHA, dA.data_ptr(), n, dB.data_ptr(), n,
                                                        BETA, dC.data_ptr(), n), 3)
            t_ven = timed(torch, lambda: torch.matmul(dB, dA), 3)
            lines.append("")
            lines.append("## phi = %g" % phi)
            lines.append("native FP64: this library's MFMA kernel %.2f ms (%.1f TFLOP/s); vendor GEMM %.2f ms (%.1f TFLOP/s)"
                         % (t_own, tf(t_own), t_ven, tf(t_ven)))
            lines.append("mode               S   ESC  ms      TFLOP/s  x vendor  guard share  (scan esc slicing gemm recompose ms)")
            for name, opt in (("unguarded 55", dict(mode=g.OZ_FIXED_UNGUARDED, max_bits=55)),
                              ("forced 55", dict(mode=g.OZ_FORCED_GUARDED, max_bits=55)),
                              ("dynamic", dict(mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200))):
                print("  %s" % name, flush=True)
                ms, res, sm = emulated(torch, g, h, n, dA, dB, dC, args.reps, **opt)
                guard = (sm["scan"] + sm["esc"] + sm["verdict"]) / ms
                lines.append("%-18s %-3d %-4d %-7.2f %-8.1f %-9.2f %-12.3f (%.2f %.2f %.2f %.2f %.2f)"
                             % (name, res.slices_used, res.esc, ms, tf(ms), t_ven / ms, guard, sm["scan"], sm["esc"],
                                sm["slicing"], sm["slice_gemm_i8"], sm["recompose"]))
            lines.append("")
            lines.append("fixed slice count, no guardrails")
            lines.append("S   pairs  ms      TFLOP/s  ms/pair  INT8 TOP/s of the slice GEMM")
            for S in range(4, 13):
                print("  S = %d" % S, flush=True)
                ms, res, sm = emulated(torch, g, h, n, dA, dB, dC, max(2, args.reps // 2), mode=g.OZ_FIXED_UNGUARDED, slices=S)
                pairs = S * (S + 1) // 2
                lines.append("%-3d %-6d %-7.2f %-8.1f %-8.3f %.0f" % (S, pairs, ms, tf(ms), ms / pairs,
                                                                     pairs * flops / (sm["slice_gemm_i8"] * 1e-3) * 1e-12))
            lines.append("")
            lines.append("block length of the coarsened ESC (dynamic mode, target 53 bits)")
            lines.append("b     ESC  S   ESC stage ms  scan ms")
            for b in (16, 32, 64, 128, 256, 1024):
                print("  b = %d" % b, flush=True)
                ms, res, sm = emulated(torch, g, h, n, dA, dB, dC, 2, mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200, esc_block=b)
                lines.append("%-5d %-4d %-3d %-13.3f %.3f" % (b, res.esc, res.slices_used, sm["esc"], sm["scan"]))
            del dA, dB, dC
            torch.cuda.empty_cache()
        path = os.path.join(OUT, "throughput_%d.txt" % n)
        with open(path, "w") as f:
            f.write("\n".join(lines) + "\n")
        print("\n".join(lines), flush=True)
    h.close()


if __name__ == "__main__":
    main()
