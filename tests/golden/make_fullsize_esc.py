"""Writes tests/golden/fullsize_esc.txt: the coarsened ESC (block length 64) of the full-size
seeded workloads, computed by the CPU oracle only (it takes minutes at these sizes, which is why
the values are stored).  Run from the repository root:  python tests/golden/make_fullsize_esc.py
"""
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ozaki as oz                              # noqa: E402
from paper_2511_13778_amd import workloads as wl            # noqa: E402

CASES = {
    # name: (generator, kwargs)
    "lognormal_4096_phi0.5_seed2": lambda: wl.lognormal_spread(4096, 4096, 4096, 0.5, seed=2),
    "lognormal_8192_phi1_seed4": lambda: wl.lognormal_spread(8192, 8192, 8192, 1.0, seed=4)[:2],
    "rowscaled_1024x1024x65536_seed6": lambda: wl.row_scaled(1024, 65536, 1024, seed=6)[:2],
    "rowscaled_32768x256x8192_seed6": lambda: wl.row_scaled(32768, 8192, 256, seed=6)[:2],
}

if __name__ == "__main__":
    only = sys.argv[1:]
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "fullsize_esc.txt")
    have = {}
    if os.path.exists(out):
        for ln in open(out):
            if ln.strip() and not ln.startswith("#"):
                k, v = ln.split()
                have[k] = int(v)
    for name, gen in CASES.items():
        if only and name not in only:
            continue
        A, B = gen()[:2]
        t0 = time.time()
        have[name] = oz.esc_coarse(A, B, 64)
        print(name, have[name], "%.0f s" % (time.time() - t0), flush=True)
        with open(out, "w") as f:
            f.write("# coarsened ESC (b = 64) of the full-size seeded workloads, written by make_fullsize_esc.py\n"
                    "# (CPU oracle only).  columns: workload esc\n")
            for k in sorted(have):
                f.write("%s %d\n" % (k, have[k]))
