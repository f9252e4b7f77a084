"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times.

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


_MODES = {"dynamic": "OZ_DYNAMIC", "forced": "OZ_FORCED_GUARDED", "unguarded": "OZ_FIXED_UNGUARDED"}
_OMODES = {"dynamic": oz.MODE_DYNAMIC, "forced": oz.MODE_FORCED_GUARDED, "unguarded": oz.MODE_FIXED_UNGUARDED}

_inputs = {}


def inputs(key, make):
    """One full-size input set at a time stays cached, so tests that share it generate it once."""
    if key not in _inputs:
        _inputs.clear()
        _inputs[key] = make()
    return _inputs[key]


def device_operands(A, B, Cin):
    key = ("dev", id(A), id(B), id(Cin))
    if key not in _inputs:
        for k_ in [k_ for k_ in _inputs if isinstance(k_, tuple) and k_[0] == "dev"]:
            del _inputs[k_]
        from paper_2511_13778_amd import ozdgemm as g
        # the host arrays are kept alongside, so their ids (the key) cannot be reused while this entry lives
        _inputs[key] = (g.to_colmajor(A), g.to_colmajor(B), None if Cin is None else g.to_colmajor(Cin),
                        oz.row_exponents(A), oz.col_exponents(B), (A, B, Cin))
    return _inputs[key][:5]


def golden_tile_esc(name):
    path = os.path.join(os.path.dirname(__file__), "golden", "tile_esc_%s.txt" % name)
    if not os.path.exists(path):
        pytest.skip("no stored per-block ESC for %s (run tests/golden/make_fullsize_esc.py)" % name)
    return np.loadtxt(path, dtype=np.int64, ndmin=2)


def sampled_parity(g, h, A, B, alpha, beta, Cin, mode, max_bits, esc_name, nsample=40, seed=0, check_bound=True,
                   infnan=False, bound_stride=3, heuristic=False, tile_esc_name=None, extra_rows=()):
    """Runs the call at full size and compares with the oracle on sampled rows and columns.  Returns
    (record, bound ratio on the sampled entries or None).  check_bound: True asserts ratio <= 1,
    "report" only returns it, False skips the exact reference."""
    m, k = A.shape
    n = B.shape[1]
    opts = g.make_opts(mode=getattr(g, _MODES[mode]), target_bits=53, max_bits=max_bits, heuristic=int(heuristic),
                       tile_slices=int(tile_esc_name is not None))
    gm = g.Gemm(h, m, n, k, opts)
    dA, dB, dC0, eA, eB = device_operands(A, B, Cin)
    dC = dC0.clone() if dC0 is not None else torch.full((n, m), float("nan"), dtype=torch.float64, device="cuda")
    gm.run(dA, m, dB, k, dC, m, alpha, beta)
    torch.cuda.synchronize()
    res = gm.result()

    tile_esc = golden_tile_esc(tile_esc_name) if tile_esc_name is not None else None
    if tile_esc is not None:
        esc = int(tile_esc.max())          # the ESC of the whole product is the largest block ESC
    else:
        esc = golden_esc(esc_name) if (mode != "unguarded" and not infnan) else -1
    hm = oz.HeuristicModel() if heuristic else None
    assert not oz.shape_only_fallback(_OMODES[mode], 53, m, n, k, hm)     # these sizes are always scanned
    v = oz.verdict(_OMODES[mode], 53, max_bits, 0, infnan, esc, m, n, k, hm, tile_esc)
    assert (res.fallback, res.reason, res.slices_used, res.esc, res.required_bits, res.infnan, res.slices_min,
            res.pair_tiles) == (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits, v.infnan, v.slices_min,
                                v.pair_tiles)
    S = v.slices_used
    S_tile = oz.tile_slices(53, tile_esc) if (tile_esc is not None and not v.fallback) else None
    if S_tile is not None:
        np.testing.assert_array_equal(gm.tile_slice_counts(), S_tile)

    rng = np.random.default_rng(seed)
    def pick(size):
        fixed = [0, 1, 255, 256, size - 257, size - 1] if size > 600 else [0, size - 1]
        rnd = rng.choice(size, min(nsample, size), replace=False).tolist()
        return np.array(sorted(set(fixed + rnd)))
    I, J = pick(m), pick(n)
    I = np.array(sorted(set(I.tolist()) | set(extra_rows)))
    Csub = None if Cin is None else Cin[np.ix_(I, J)]
    got = dC.index_select(0, torch.as_tensor(J, device="cuda")).index_select(1, torch.as_tensor(I, device="cuda"))
    got = got.cpu().numpy().T

    if not v.fallback:
        gA, gB = gm.row_exponents()
        np.testing.assert_array_equal(gA, eA)
        np.testing.assert_array_equal(gB, eB)
        As = oz.slice_rows(A[I], eA[I], S)
        Bs = oz.slice_rows(np.ascontiguousarray(B[:, J].T), eB[J], S)
        gAs, gBs = gm.slices_sampled(S, I, J)
        np.testing.assert_array_equal(gAs, As)
        np.testing.assert_array_equal(gBs, Bs)
        P = oz.slice_products(As, Bs)
        # the slice GEMM leaves the anti-diagonal sums of a k-block aggregated: leading word + balanced digits
        gT, glo = gm.digits_sampled(S, P.shape[0], I, J)
        if S_tile is None:
            T0, lo = oz.normalised_digits(P)
            np.testing.assert_array_equal(gT, T0)
            np.testing.assert_array_equal(glo, lo)
            want = oz.axpby(alpha, oz.recompose(P, eA[I], eB[J]), beta, Csub)
        else:
            # every sampled entry belongs to a block with its own count: it walked the anti-diagonals
            # below that count only, and is aggregated and recomposed from those
            S_el = S_tile[np.ix_(I // oz.TILE, J // oz.TILE)]
            want = np.empty((len(I), len(J)))
            for St in np.unique(S_el):
                sel = S_el == St
                T0, lo = oz.normalised_digits(P[:, :St])
                np.testing.assert_array_equal(gT[:, sel], T0[:, sel])
                np.testing.assert_array_equal(glo[:, :St - 1][:, :, sel], lo[:, :, sel])
                want[sel] = oz.axpby(alpha, oz.recompose(P[:, :St], eA[I], eB[J]), beta, Csub)[sel]
        np.testing.assert_array_equal(got, want)
    del gm, dC

    if not check_bound:
        return res, None
    idx = [(a, b) for a in range(0, len(I), bound_stride) for b in range(0, len(J), bound_stride)]
    exact = ex.exact_entries(A[I], B[:, J], idx, alpha, beta, Csub)
    den = ex.bound_denominator(A[I], B[:, J], idx, alpha, beta, Csub)
    ratio = ex.gradeA_ratio(np.array([got[a, b] for a, b in idx]), exact, den, k)
    if check_bound is True:
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
    A, B, Cin = inputs("ln8192phi1", lambda: wl.lognormal_spread(8192, 8192, 8192, 1.0, seed=4, with_c=True))
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "forced", 55, "lognormal_8192_phi1_seed4")
    assert res.slices_used == 7 and res.fallback == 0


def test_headline_8192_dynamic(lib):
    g, h = lib
    A, B, Cin = inputs("ln8192phi1", lambda: wl.lognormal_spread(8192, 8192, 8192, 1.0, seed=4, with_c=True))
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "dynamic", 200, "lognormal_8192_phi1_seed4", nsample=24)
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, res.esc)


def test_headline_8192_as_shipped_goes_native_after_the_esc(lib):
    # the default options (OZ_DYNAMIC, run-time heuristic on): the operands are scanned, the ESC is
    # computed and reported, and the cost model then sends the nine-slice job to the native FP64 GEMM
    g, h = lib
    A, B, Cin = inputs("ln8192phi1", lambda: wl.lognormal_spread(8192, 8192, 8192, 1.0, seed=4, with_c=True))
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "dynamic", 200, "lognormal_8192_phi1_seed4", nsample=24,
                                heuristic=True)
    assert (res.fallback, res.reason, res.slices_used, res.infnan) == (1, oz.REASON_HEURISTIC, 0, 0)
    assert res.esc == golden_esc("lognormal_8192_phi1_seed4") and res.required_bits == 53 + res.esc


def test_per_tile_slice_counts_8192_localised_hard_rows(lib):
    # 100 difficult rows in an otherwise uniform 8192^3 product: with one slice count for all of C the ESC
    # of those rows sets S for all 1024 blocks; with per-block counts only the two block rows they cross pay
    g, h = lib
    A, B = inputs("widerows8192", lambda: wl.wide_rows(8192, 8192, 8192, seed=11, row_lo=3000, row_hi=3100, spread=24))
    res, ratio = sampled_parity(g, h, A, B, 1.0, 0.0, None, "dynamic", 200, None, nsample=30,
                                tile_esc_name="widerows_8192_seed11", extra_rows=(2999, 3000, 3050, 3071, 3072, 3099, 3100))
    nt = 32 * 32
    assert res.fallback == 0 and res.slices_min == 7 and res.slices_used >= 10
    assert res.pair_tiles == 64 * oz.pairs_of(res.slices_used) + (nt - 64) * oz.pairs_of(7)
    assert res.pair_tiles * 1.8 < nt * oz.pairs_of(res.slices_used)


def test_config3_8192_small_spread_dynamic(lib):
    # phi = 0.1: nearly uniform exponents, the ESC adds one slice to the seven of 53 bits
    g, h = lib
    A, B, Cin = inputs("ln8192phi0.1", lambda: wl.lognormal_spread(8192, 8192, 8192, 0.1, seed=3, with_c=True))
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "dynamic", 200, "lognormal_8192_phi0.1_seed3", nsample=24)
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, res.esc) == 8


def test_config3_8192_wide_spread_dynamic_and_forced(lib):
    # phi = 2: exponents inside a row spread over tens of bits.  DYNAMIC raises the slice count and
    # meets the bound.  FORCED to 55 bits runs its seven slices whatever the ESC says (only Inf/NaN
    # makes it yield), stays bit-identical to the oracle, reports required_bits far above 55, and
    # loses the componentwise bound on some entries: the bound is a property of the input in that
    # mode (solid lines of the paper's Test-2 figure; its remark on QR residuals with fixed 55 bits).
    g, h = lib
    A, B, Cin = inputs("ln8192phi2", lambda: wl.lognormal_spread(8192, 8192, 8192, 2.0, seed=5, with_c=True))
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "dynamic", 200, "lognormal_8192_phi2_seed5", nsample=24)
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, res.esc) == 11
    res, ratio = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "forced", 55, "lognormal_8192_phi2_seed5", nsample=24,
                                check_bound="report", bound_stride=1)
    assert res.fallback == 0 and res.slices_used == 7 and res.required_bits > 55
    assert ratio > 1.0, ratio


def test_config3_16384_forced_and_dynamic(lib):
    g, h = lib
    A, B, Cin = inputs("ln16384phi1", lambda: wl.lognormal_spread(16384, 16384, 16384, 1.0, seed=4, with_c=True))
    res, _ = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "forced", 55, "lognormal_16384_phi1_seed4", nsample=24)
    assert res.fallback == 0 and res.slices_used == 7
    res, _ = sampled_parity(g, h, A, B, 1.5, 0.5, Cin, "dynamic", 200, "lognormal_16384_phi1_seed4", nsample=16)
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, res.esc) >= 8


def test_config5_2048_wide_span_falls_back(lib):
    # every entry N(0,1) * 2^-300 or 2^+300: the coarsened ESC is in the hundreds, beyond any cap
    g, h = lib
    A, B = inputs("wide2048", lambda: wl.wide_span(2048, 2048, 2048, seed=7))
    for max_bits in (55, 200):
        res, ratio = sampled_parity(g, h, A, B, 1.0, 0.0, None, "dynamic", max_bits, "widespan_2048_seed7", nsample=24)
        assert (res.fallback, res.reason, res.slices_used) == (1, oz.REASON_BITS, 0) and res.esc > 600


def test_config5_2048_inf_nan_falls_back(lib):
    g, h = lib
    def make():
        A0, B0 = wl.lognormal_spread(2048, 2048, 2048, 0.5, seed=8)
        return wl.plant_inf_nan(A0, B0, seed=8)
    A, B = inputs("infnan2048", make)
    for mode, max_bits in (("dynamic", 200), ("dynamic", 55), ("forced", 55)):
        res, _ = sampled_parity(g, h, A, B, 1.0, 0.0, None, mode, max_bits, None, check_bound=False, infnan=True)
        assert (res.fallback, res.reason, res.infnan, res.esc) == (1, oz.REASON_INFNAN, 1, -1)
    # the native path's result: special values where an FP64 GEMM puts them, finite entries inside the bound
    opts = g.make_opts(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0)
    gm = g.Gemm(h, 2048, 2048, 2048, opts)
    dA, dB = g.to_colmajor(A), g.to_colmajor(B)
    dC = torch.empty((2048, 2048), dtype=torch.float64, device="cuda")
    gm.run(dA, 2048, dB, 2048, dC, 2048)
    torch.cuda.synchronize()
    got = g.from_colmajor(dC)
    with np.errstate(all="ignore"):
        ref = A @ B
    np.testing.assert_array_equal(np.isnan(got), np.isnan(ref))
    np.testing.assert_array_equal(np.isposinf(got), np.isposinf(ref))
    np.testing.assert_array_equal(np.isneginf(got), np.isneginf(ref))
    fin = np.argwhere(np.isfinite(ref))
    pick = fin[np.random.default_rng(8).choice(len(fin), 300, replace=False)]
    idx = [(int(i), int(j)) for i, j in pick]
    ratio = ex.gradeA_ratio(np.array([got[i, j] for i, j in idx]), ex.exact_entries(A, B, idx),
                            ex.bound_denominator(A, B, idx), 2048)
    assert ratio <= 1.0, ratio


def test_config5_2048_rank1_cancellation(lib):
    # A = u v^T + 1e-12 noise: products cancel heavily; the ESC raises S and the bound holds; with a cap
    # of 55 bits the same ESC sends the call to the native path
    g, h = lib
    A, B = inputs("rank1_2048", lambda: wl.rank1_cancel(2048, 2048, 2048, seed=9))
    res, ratio = sampled_parity(g, h, A, B, 1.0, 0.0, None, "dynamic", 200, "rank1_2048_seed9", nsample=24)
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, res.esc) >= 8
    res, ratio = sampled_parity(g, h, A, B, 1.0, 0.0, None, "dynamic", 55, "rank1_2048_seed9", nsample=24)
    assert (res.fallback, res.reason) == (1, oz.REASON_BITS)


def test_config4_short_k_forced_and_dynamic(lib):
    # 16384 x 16384 x 512: eight ESC blocks, two K tiles of the slice GEMM per pair, 4096 output tiles
    g, h = lib
    A, B, _ = inputs("rs16384x512", lambda: wl.row_scaled(16384, 512, 16384, seed=6))
    res, _ = sampled_parity(g, h, A, B, 1.0, 0.0, None, "forced", 55, "rowscaled_16384x16384x512_seed6", nsample=24)
    assert res.slices_used == 7 and res.fallback == 0
    res, _ = sampled_parity(g, h, A, B, 1.0, 0.0, None, "dynamic", 200, "rowscaled_16384x16384x512_seed6", nsample=24)
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
    A, B, _ = inputs("rs16384x512", lambda: wl.row_scaled(16384, 512, 16384, seed=6))
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


@pytest.mark.parametrize("tall", [True, False])
def test_largest_m_and_n(lib, tall):
    # m, then n, at the library's limit (2^22): a strip of 16384 x 2 tiles of C, 64 rounds of the slice
    # GEMM's workgroups, element offsets past 2^31 and byte offsets past 2^32 inside the leading-word and
    # digit planes, and 65536-wide launches of the scan, slicing and recomposition kernels
    g, h = lib
    if tall:
        A, B = wl.lognormal_spread(1 << 22, 24, 300, 1.0, seed=26)
        name = "lognormal_4194304x300x24_seed26"
    else:
        A, B = wl.lognormal_spread(300, 24, 1 << 22, 1.0, seed=27)
        name = "lognormal_300x4194304x24_seed27"
    res, ratio = sampled_parity(g, h, A, B, 1.0, 0.0, None, "dynamic", 200, name, nsample=40)
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, res.esc) == 10
    _inputs.clear()
    torch.cuda.empty_cache()


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
