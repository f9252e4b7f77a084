"""GPU parity at BASELINE's full sizes, in the launch configuration bench.py times.

The oracle cannot run 8192^3 in full, so it is evaluated on sampled rows of op(A) and columns of
op(B) (first, last and random ones, so that many tiles and both tile edges are hit): row/column
exponents are compared in full, slices for the sampled rows/columns, anti-diagonal products and
the final C for every sampled (row, column) pair, all bit-exact; the componentwise bound is checked
against the exact reference on the same pairs.  The full-size ESC comes from tests/golden (written
by make_fullsize_esc.py, which calls only the oracle).
"""
import os

import numpy as np
import pytest

from oracle import exact as ex
from oracle import ozaki as oz
from paper_2511_13778_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

GOLD = os.path.join(os.path.dirname(__file__), "golden", "fullsize_esc.txt")


def golden_esc(name):
    for ln in open(GOLD):
        if ln.strip() and not ln.startswith("#"):
            k, v = ln.split()
            if k == name:
                return int(v)
    pytest.skip("no stored ESC for %s (run tests/golden/make_fullsize_esc.py)" % name)


@pytest.fixture(scope="module")
def lib():
    from paper_2511_13778_amd import ozdgemm as g
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
    h = g.Handle(0)
    yield g, h
    h.close()


def sampled_parity(g, h, A, B, alpha, beta, Cin, mode, max_bits, esc_name, nsample=40, seed=0, check_bound=True):
    m, k = A.shape
    n = B.shape[1]
    opts = g.make_opts(mode={"dynamic": g.OZ_DYNAMIC, "forced": g.OZ_FORCED_GUARDED,
                             "unguarded": g.OZ_FIXED_UNGUARDED}[mode],
                       target_bits=53, max_bits=max_bits, heuristic=0)
    gm = g.Gemm(h, m, n, k, opts)
    dA, dB = g.to_colmajor(A), g.to_colmajor(B)
    dC = g.to_colmajor(Cin) if Cin is not None else torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda")
    gm.run(dA, m, dB, k, dC, m, alpha, beta)
    torch.cuda.synchronize()
    res = gm.result()

    esc = golden_esc(esc_name) if mode != "unguarded" else -1
    v = oz.verdict({"dynamic": oz.MODE_DYNAMIC, "forced": oz.MODE_FORCED_GUARDED,
                    "unguarded": oz.MODE_FIXED_UNGUARDED}[mode], 53, max_bits, 0, False, esc, m, n, k)
    assert (res.fallback, res.reason, res.slices_used, res.esc, res.required_bits) == \
           (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits)
    S = v.slices_used

    eA, eB = oz.row_exponents(A), oz.col_exponents(B)
    gA, gB = gm.row_exponents()
    np.testing.assert_array_equal(gA, eA)
    np.testing.assert_array_equal(gB, eB)

    rng = np.random.default_rng(seed)
    def pick(size):
        fixed = [0, 1, 255, 256, size - 257, size - 1] if size > 600 else [0, size - 1]
        rnd = rng.choice(size, min(nsample, size), replace=False).tolist()
        return np.array(sorted(set(fixed + rnd)))
    I, J = pick(m), pick(n)
    As = oz.slice_rows(A[I], eA[I], S)
    Bs = oz.slice_rows(np.ascontiguousarray(B[:, J].T), eB[J], S)
    gAs, gBs = gm.slices_sampled(S, I, J)
    np.testing.assert_array_equal(gAs, As)
    np.testing.assert_array_equal(gBs, Bs)
    P = oz.slice_products(As, Bs)
    np.testing.assert_array_equal(gm.products_sampled(S, P.shape[0], I, J), P)
    Csub = None if Cin is None else Cin[np.ix_(I, J)]
    want = oz.axpby(alpha, oz.recompose(P, eA[I], eB[J]), beta, Csub)
    got = dC.index_select(0, torch.as_tensor(J, device="cuda")).index_select(1, torch.as_tensor(I, device="cuda"))
    got = got.cpu().numpy().T
    np.testing.assert_array_equal(got, want)

    if not check_bound:
        return res, None
    idx = [(a, b) for a in range(0, len(I), 3) for b in range(0, len(J), 3)]
    exact = ex.exact_entries(A[I], B[:, J], idx, alpha, beta, Csub)
    den = ex.bound_denominator(A[I], B[:, J], idx, alpha, beta, Csub)
    ratio = ex.gradeA_ratio(np.array([got[a, b] for a, b in idx]), exact, den, k)
    assert ratio <= 1.0, ratio
    return res, ratio


def test_config2_4096_dynamic(lib):
    g, h = lib
    A, B = wl.lognormal_spread(4096, 4096, 4096, 0.5, seed=2)
    res, ratio = sampled_parity(g, h, A, B, 1.0, 0.0, None, "dynamic", 200, "lognormal_4096_phi0.5_seed2")
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, res.esc)


def test_headline_8192_forced_55(lib):
    # the benchmark's own configuration
    g, h = lib
    A, B, Cin = wl.lognormal_spread(8192, 8192, 8192, 1.0, seed=4, with_c=True)
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "forced", 55, "lognormal_8192_phi1_seed4")
    assert res.slices_used == 7 and res.fallback == 0


def test_headline_8192_dynamic(lib):
    g, h = lib
    A, B, Cin = wl.lognormal_spread(8192, 8192, 8192, 1.0, seed=4, with_c=True)
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "dynamic", 200, "lognormal_8192_phi1_seed4", nsample=24)
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, res.esc)


def test_config4_long_k_four_kblocks(lib):
    # k = 65536 needs four int32 k-blocks at S = 7; rows of A scaled by 2^(i mod 40)
    g, h = lib
    A, B, _ = wl.row_scaled(1024, 65536, 1024, seed=6)
    res, ratio = sampled_parity(g, h, A, B, 1.0, 0.0, None, "forced", 55, "rowscaled_1024x1024x65536_seed6")
    assert res.slices_used == 7


def test_config4_tall_skinny(lib):
    g, h = lib
    A, B, _ = wl.row_scaled(32768, 8192, 256, seed=6)
    sampled_parity(g, h, A, B, 1.0, 0.0, None, "forced", 55, "rowscaled_32768x256x8192_seed6")


def test_config4_short_k_unguarded(lib):
    g, h = lib
    A, B, _ = wl.row_scaled(16384, 512, 16384, seed=6)
    sampled_parity(g, h, A, B, 1.0, 0.0, None, "unguarded", 55, None)


def test_many_tiles_long_k(lib):
    # 18 x 18 = 324 tiles of 256 x 256: more than the 256 workgroups the chip runs at a time, so the
    # slice GEMM's workgroups take the in-step waits (a full round of 32 per XCD and a partial one),
    # and k = 12288 adds the waits after every anti-diagonal
    g, h = lib
    A, B, Cin = wl.lognormal_spread(4608, 12288, 4608, 1.0, seed=23, with_c=True)
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "unguarded", 55, None, nsample=32)
    assert res.slices_used == 7


def test_longest_k(lib):
    # k at the library's limit (2^21): 113 int32 k-blocks, one tile split into 256 parts along k
    g, h = lib
    A, B = wl.uniform_pm1(8, 1 << 21, 12, seed=25)
    res, _ = sampled_parity(g, h, A, B, 1.0, 0.0, None, "unguarded", 55, None, check_bound=False)
    assert res.slices_used == 7


def test_reproducible_across_calls(lib):
    # integer accumulation is order-free and the FP64 order is fixed: C is bit-identical run to run
    g, h = lib
    A, B = wl.lognormal_spread(2048, 2048, 2048, 1.0, seed=21)
    opts = g.make_opts(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0)
    gm = g.Gemm(h, 2048, 2048, 2048, opts)
    dA, dB = g.to_colmajor(A), g.to_colmajor(B)
    outs = []
    for _ in range(3):
        dC = torch.empty((2048, 2048), dtype=torch.float64, device="cuda")
        gm.run(dA, 2048, dB, 2048, dC, 2048)
        torch.cuda.synchronize()
        outs.append(dC.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])
