"""Writes tests/golden/fullsize_esc.txt: the coarsened ESC (block length 64) of the full-size
seeded workloads, computed by the CPU oracle only (it takes minutes at these sizes, which is why
the values are stored).  Run from the repository root:

    python tests/golden/make_fullsize_esc.py [workload ...]

The ESC is 1 + a maximum over all (row of A, column of B) pairs, clamped; so the oracle is called
on slabs of rows of A (each against the whole of B) and the slab results are combined with max():
the same number as one call on the whole matrices, in bounded memory and on several host cores.
"""
import os
import sys
import time
from concurrent.futures import ProcessPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ozaki as oz                              # noqa: E402
from paper_2511_13778_amd import workloads as wl            # noqa: E402

CASES = {
    # name: generator of (A, B)
    "lognormal_4096_phi0.5_seed2": lambda: wl.lognormal_spread(4096, 4096, 4096, 0.5, seed=2),
    "lognormal_8192_phi0.1_seed3": lambda: wl.lognormal_spread(8192, 8192, 8192, 0.1, seed=3)[:2],
    "lognormal_8192_phi1_seed4": lambda: wl.lognormal_spread(8192, 8192, 8192, 1.0, seed=4)[:2],
    "lognormal_8192_phi2_seed5": lambda: wl.lognormal_spread(8192, 8192, 8192, 2.0, seed=5)[:2],
    "lognormal_16384_phi1_seed4": lambda: wl.lognormal_spread(16384, 16384, 16384, 1.0, seed=4)[:2],
    "rowscaled_1024x1024x65536_seed6": lambda: wl.row_scaled(1024, 65536, 1024, seed=6)[:2],
    "rowscaled_32768x256x8192_seed6": lambda: wl.row_scaled(32768, 8192, 256, seed=6)[:2],
    "rowscaled_16384x16384x512_seed6": lambda: wl.row_scaled(16384, 512, 16384, seed=6)[:2],
    "widespan_2048_seed7": lambda: wl.wide_span(2048, 2048, 2048, seed=7),
    "rank1_2048_seed9": lambda: wl.rank1_cancel(2048, 2048, 2048, seed=9),
    # m, then n, at the library's limit of 2^22
    "lognormal_4194304x300x24_seed26": lambda: wl.lognormal_spread(1 << 22, 24, 300, 1.0, seed=26),
    "lognormal_300x4194304x24_seed27": lambda: wl.lognormal_spread(300, 24, 1 << 22, 1.0, seed=27),
}

# workloads whose per-block ESC table (256 x 256 blocks of C) is stored, one file each:
# tile_esc_<name>.txt, row ti = the ESCs of blocks (ti, 0..)
TILE_CASES = {
    "widerows_8192_seed11": lambda: wl.wide_rows(8192, 8192, 8192, seed=11, row_lo=3000, row_hi=3100, spread=24),
}

SLAB_ELEMS = 1 << 24          # (rows of a slab) x n: bounds the oracle's m x n temporaries
WORKERS = int(os.environ.get("ESC_WORKERS", "4"))

_A = _B = None                # inherited by the forked workers


def _slab(r):
    return oz.esc_coarse(_A[r[0]:r[1]], _B, 64)


def _tile_slab(r):
    return oz.esc_coarse_tiles(_A[r[0]:r[1]], _B, 64, oz.TILE)


def tile_esc_by_slabs(A, B):
    """esc_coarse_tiles on slabs of whole block rows (a block's ESC only involves its own rows of A)."""
    global _A, _B
    _A, _B = A, B
    m, n = A.shape[0], B.shape[1]
    rows = max(oz.TILE, min(m, SLAB_ELEMS // n) // oz.TILE * oz.TILE)
    slabs = [(r0, min(m, r0 + rows)) for r0 in range(0, m, rows)]
    with ProcessPoolExecutor(max_workers=min(WORKERS, len(slabs))) as pool:
        parts = list(pool.map(_tile_slab, slabs))
    import numpy as np
    return np.vstack(parts)


def esc_by_slabs(A, B):
    global _A, _B
    _A, _B = A, B
    m, n = A.shape[0], B.shape[1]
    rows = max(1, min(m, SLAB_ELEMS // n))
    slabs = [(r0, min(m, r0 + rows)) for r0 in range(0, m, rows)]
    if len(slabs) == 1:
        return _slab(slabs[0])
    with ProcessPoolExecutor(max_workers=min(WORKERS, len(slabs))) as pool:
        return max(pool.map(_slab, slabs))


if __name__ == "__main__":
    only = sys.argv[1:]
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "fullsize_esc.txt")
    have = {}
    if os.path.exists(out):
        for ln in open(out):
            if ln.strip() and not ln.startswith("#"):
                k, v = ln.split()
                have[k] = int(v)
    here = os.path.dirname(os.path.abspath(__file__))
    for name, gen in TILE_CASES.items():
        if only and name not in only:
            continue
        A, B = gen()[:2]
        t0 = time.time()
        T = tile_esc_by_slabs(A, B)
        print(name, "blocks", T.shape, "ESC values", sorted(set(T.ravel().tolist())), "%.0f s" % (time.time() - t0), flush=True)
        with open(os.path.join(here, "tile_esc_%s.txt" % name), "w") as f:
            f.write("# coarsened ESC (b = 64) of every 256 x 256 block of C, written by make_fullsize_esc.py\n"
                    "# (CPU oracle only).  line ti = blocks (ti, 0), (ti, 1), ...\n")
            for row in T:
                f.write(" ".join(str(int(v)) for v in row) + "\n")
    for name, gen in CASES.items():
        if only and name not in only:
            continue
        A, B = gen()[:2]
        t0 = time.time()
        have[name] = esc_by_slabs(A, B)
        print(name, have[name], "%.0f s" % (time.time() - t0), flush=True)
        with open(out, "w") as f:
            f.write("# coarsened ESC (b = 64) of the full-size seeded workloads, written by make_fullsize_esc.py\n"
                    "# (CPU oracle only).  columns: workload esc\n")
            for k in sorted(have):
                f.write("%s %d\n" % (k, have[k]))
