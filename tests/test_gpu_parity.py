"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: bit-exact for row/column exponents, ESC, slice count, fallback flag, slices (int8) and
anti-diagonal products (int32); final C within k*2^-53 * (|alpha||A||B| + |beta||C|)
componentwise of the exact reference, and (because the library uses the oracle's summation
order) also bit-identical to the oracle's C on the emulated path.
"""
import numpy as np
import pytest

from oracle import exact as ex
from oracle import ozaki as oz
from paper_2511_13778_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def lib():
    from paper_2511_13778_amd import ozdgemm as g
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
    h = g.Handle(0)
    yield g, h
    h.close()


def run_gpu(g, h, A, B, alpha=1.0, beta=0.0, Cin=None, transa="N", transb="N", pad=0, **opt):
    """Runs oz_dgemm on logical A (m x k), B (k x n); returns (C, Gemm object, Result)."""
    m, k = A.shape
    n = B.shape[1]
    opts = g.make_opts(**opt)
    gm = g.Gemm(h, m, n, k, opts, transa, transb)

    def dev(X, trans):
        # column-major storage of X (or of X^T when trans), leading dimension padded by `pad`
        S = X.T if trans == "T" else X
        rows, cols = S.shape
        ld = max(1, rows) + pad
        buf = np.full((cols, ld), 7.25)           # padding holds junk that must never be read as data
        buf[:, :rows] = S.T
        return torch.from_numpy(buf).cuda(), ld

    dA, lda = dev(A, transa)
    dB, ldb = dev(B, transb)
    ldc = max(1, m) + pad
    cbuf = np.full((n, ldc), np.nan)              # NaN: proves C is not read when beta == 0
    if Cin is not None:
        cbuf[:, :m] = Cin.T
    dC = torch.from_numpy(cbuf).cuda()
    gm.run(dA, lda, dB, ldb, dC, ldc, alpha, beta)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    if pad:
        assert np.all(np.isnan(out[:, m:])), "wrote outside the m x n window of C"
    return out[:, :m].T.copy(), gm, gm.result()


MODES = {"dynamic": oz.MODE_DYNAMIC, "forced": oz.MODE_FORCED_GUARDED, "fixed_guarded": oz.MODE_FIXED_GUARDED,
         "unguarded": oz.MODE_FIXED_UNGUARDED, "native": oz.MODE_NATIVE}


def check_against_oracle(g, h, A, B, alpha=1.0, beta=0.0, Cin=None, mode="forced", target_bits=53,
                         max_bits=55, slices=0, esc_block=0, transa="N", transb="N", pad=0, bound=True,
                         intermediates=True):
    m, k = A.shape
    n = B.shape[1]
    got, gm, res = run_gpu(g, h, A, B, alpha, beta, Cin, transa, transb, pad, mode=MODES[mode],
                           target_bits=target_bits, max_bits=max_bits, slices=slices, esc_block=esc_block,
                           heuristic=0)
    tr = oz.emulated_dgemm(A, B, alpha, beta, Cin, mode=MODES[mode], target_bits=target_bits,
                           max_bits=max_bits, slices=slices, esc_block=esc_block or oz.DEFAULT_ESC_BLOCK)
    v = tr.verdict
    assert (res.fallback, res.reason, res.slices_used, res.esc, res.required_bits, res.infnan, res.slices_min,
            res.pair_tiles) == (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits, v.infnan, v.slices_min,
                                v.pair_tiles)
    if not v.fallback:
        S = v.slices_used
        if intermediates:
            eA, eB = gm.row_exponents()
            np.testing.assert_array_equal(eA, np.where(tr.eA > oz.NEG_INF_BELOW, tr.eA, -12288))
            np.testing.assert_array_equal(eB, np.where(tr.eB > oz.NEG_INF_BELOW, tr.eB, -12288))
            As, Bs = gm.slices(S)
            np.testing.assert_array_equal(As, tr.As)
            np.testing.assert_array_equal(Bs, tr.Bs)
            # the slice GEMM leaves the anti-diagonal sums of a k-block aggregated (leading word + balanced digits)
            T0, lo = oz.normalised_digits(tr.P)
            gT, glo = gm.digits(S, tr.P.shape[0])
            np.testing.assert_array_equal(gT, T0)
            np.testing.assert_array_equal(glo, lo)
        np.testing.assert_array_equal(got, tr.C)          # same summation order: bit-identical
    else:
        # native path: any value inside the bound is correct; compare with the host product wherever that is finite
        with np.errstate(all="ignore"):
            slack = 2.0 * (k + 2) * 2.0 ** -53 * (abs(alpha) * (np.abs(A) @ np.abs(B)) +
                                                  (abs(beta) * np.abs(Cin) if (Cin is not None and beta != 0.0) else 0.0))
            fin = np.isfinite(tr.C) & np.isfinite(slack)
            assert np.all(np.abs(got[fin] - tr.C[fin]) <= slack[fin])
    if bound:
        idx = [(i, j) for i in range(m) for j in range(n)]
        if len(idx) > 6000:                       # exact reference on a seeded sample of the entries
            pick = np.random.default_rng(m * 31 + n).choice(len(idx), 6000, replace=False)
            idx = [idx[t] for t in pick]
        exact = ex.exact_entries(A, B, idx, alpha, beta, Cin)
        den = ex.bound_denominator(A, B, idx, alpha, beta, Cin)
        assert ex.gradeA_ratio(np.array([got[i, j] for i, j in idx]), exact, den, k) <= 1.0
    return got, res, tr


def test_config1_128_cubed(lib):
    g, h = lib
    A, B = wl.uniform_pm1(128, 128, 128, seed=1)
    for mode in ("unguarded", "forced"):
        _, res, _ = check_against_oracle(g, h, A, B, mode=mode, max_bits=55)
        assert res.slices_used == 7 and res.fallback == 0


def test_ragged_multi_tile_dynamic(lib):
    # several 256-tiles in both directions, ragged tails in m, n and k
    g, h = lib
    A, B, Cin = wl.lognormal_spread(300, 777, 520, 1.0, seed=3, with_c=True)
    _, res, _ = check_against_oracle(g, h, A, B, 1.5, 0.5, Cin, mode="dynamic", max_bits=200, pad=3)
    assert res.fallback == 0 and res.slices_used >= 8


@pytest.mark.parametrize("ta,tb", [("N", "N"), ("T", "N"), ("N", "T"), ("T", "T")])
def test_transposes(lib, ta, tb):
    g, h = lib
    A, B = wl.lognormal_spread(130, 200, 260, 0.5, seed=11)
    check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200, transa=ta, transb=tb, pad=5)


def test_alpha_beta_round_separately(lib):
    # alpha and beta that are not powers of two: alpha*AB and beta*C are rounded on their own and then
    # added (no fused multiply-add), which is what the oracle does; a fused epilogue differs in the last bit
    g, h = lib
    A, B, Cin = wl.lognormal_spread(257, 300, 130, 0.5, seed=33, with_c=True)
    check_against_oracle(g, h, A, B, 1.1, 0.3, Cin, mode="forced", max_bits=55, pad=1)
    check_against_oracle(g, h, A, B, -0.7, 1.9, Cin, mode="dynamic", max_bits=200, transa="T")


def test_int32_k_blocking(lib):
    # S = 7 takes 18688 k per int32 accumulator: 19000 needs two k-blocks
    g, h = lib
    A, B = wl.uniform_pm1(40, 19000, 24, seed=12)
    _, res, tr = check_against_oracle(g, h, A, B, mode="unguarded", max_bits=55, bound=False)
    assert tr.P.shape[0] == 2
    idx = [(i, j) for i in range(0, 40, 7) for j in range(0, 24, 5)]
    exact = ex.exact_entries(A, B, idx)
    den = ex.bound_denominator(A, B, idx)
    got = np.array([_[i, j] for i, j in idx])
    assert ex.gradeA_ratio(got, exact, den, 19000) <= 1.0


def test_worst_case_digits_do_not_overflow_int32(lib):
    # every digit of every slice at an extreme of its range, longest k-block
    g, h = lib
    S = 3
    k = oz.k_block_length(S)
    a = -4161664.0                  # q = 0: X = -63*65536 - 128*256 - 128, digits (-63, -128, -128)
    A = np.full((4, k), a)
    B = np.full((k, 4), a)
    check_against_oracle(g, h, A, B, mode="unguarded", slices=S, bound=False)


@pytest.mark.parametrize("S", [1, 2, 9, 12, 26])
def test_slice_counts_beyond_64_bits(lib, S):
    g, h = lib
    rng = np.random.default_rng(S)
    A = rng.standard_normal((20, 70)) * np.exp2(rng.integers(-30, 30, (20, 70)))
    B = rng.standard_normal((70, 12)) * np.exp2(rng.integers(-30, 30, (70, 12)))
    A[3, 5] = 5e-324
    A[4, :] = np.ldexp(rng.uniform(-1, 1, 70), -1060)
    check_against_oracle(g, h, A, B, mode="unguarded", slices=S, bound=False)


def test_zeros_and_negative_zero(lib):
    g, h = lib
    rng = np.random.default_rng(5)
    A = rng.standard_normal((70, 200))
    B = rng.standard_normal((200, 90))
    A[10, :] = 0.0                   # all-zero row
    B[:, 20] = 0.0                   # all-zero column
    A[:, 64:128] = 0.0               # a whole ESC block of zeros in every row
    A[5, 3] = -0.0
    B[7, 7] = -0.0
    got, res, _ = check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200)
    assert res.fallback == 0
    assert np.all(got[10, :] == 0.0) and np.all(got[:, 20] == 0.0)
    assert not np.any(np.signbit(got[10, :]))


def test_denormal_inputs(lib):
    # every entry of A denormal (true exponents from the leading bit, no implicit one); the
    # product lands in the normal range again.  Slices and products must match the oracle; the
    # result must be the exact product up to the usual bound.
    g, h = lib
    rng = np.random.default_rng(15)
    A = np.ldexp(rng.uniform(-1, 1, (40, 96)), -1040)
    A[0, 0] = 5e-324
    B = np.ldexp(rng.uniform(-1, 1, (96, 30)), 900)
    assert np.all(np.abs(A) < 2.3e-308)
    got, res, _ = check_against_oracle(g, h, A, B, mode="forced", max_bits=55)
    assert res.fallback == 0 and res.esc < 40


def test_zero_blocks_identically_zero_product(lib):
    g, h = lib
    A = np.hstack([np.full((8, 64), 3.0), np.zeros((8, 64))])
    B = np.vstack([np.zeros((64, 8)), np.full((64, 8), 5.0)])
    got, res, _ = check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200)
    assert res.esc == 1 and np.all(got == 0.0)
    # one zero in each operand's only block: no candidate, ESC unbounded -> native path
    A2 = np.ones((4, 64)); A2[:, 0] = 0.0
    B2 = np.ones((64, 4)); B2[1, :] = 0.0
    got, res, _ = check_against_oracle(g, h, A2, B2, mode="dynamic", max_bits=200)
    assert (res.fallback, res.reason, res.esc) == (1, oz.REASON_BITS, oz.ESC_CAP)
    assert np.all(got == 62.0)


@pytest.mark.parametrize("b", [16, 128, 1024])
def test_esc_block_lengths(lib, b):
    g, h = lib
    A, B = wl.lognormal_spread(64, 1100, 64, 1.5, seed=20 + b)
    check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200, esc_block=b, intermediates=False)


@pytest.mark.parametrize("span", [30, 36, 37, 38, 39, 45, 70])
def test_esc_across_matrix_unit_range(lib, span):
    # One dot product whose best block candidate sits `span` bits below eA + eB: spans up to 37 are
    # resolved by the matrix-unit ESC kernel, larger ones by the int16 kernel; both must be exact.
    g, h = lib
    rng = np.random.default_rng(span)
    m, k, n = 70, 200, 150
    A = rng.uniform(0.5, 1.0, (m, k)) * rng.choice([-1.0, 1.0], (m, k))
    B = rng.uniform(0.5, 1.0, (k, n)) * rng.choice([-1.0, 1.0], (k, n))
    i, j = 66, 131                                   # in the last 32x32 tile of each direction
    A[i, 1:] *= 2.0 ** -span
    B[0, j] *= 2.0 ** -span
    B[2:, j] *= 2.0 ** -span
    _, res, tr = check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200, bound=False,
                                      intermediates=False)
    assert res.esc == span + 1 and res.fallback == 0


def test_fixed_guarded_trips_where_its_slices_run_out(lib):
    # "55 bits" are seven slices, which carry 54 magnitude bits beside the headroom bit: with ESC = 1 the
    # fixed-and-guarded mode emulates (53 + 1 = 54), with ESC = 2 (required_bits == max_bits == 55) it
    # must already fall back, exactly where the dynamic rule moves to eight slices
    g, h = lib
    rng = np.random.default_rng(3)
    m, k, n = 40, 96, 50
    A = rng.uniform(0.5, 1.0, (m, k)) * rng.choice([-1.0, 1.0], (m, k))
    B = rng.uniform(0.5, 1.0, (k, n)) * rng.choice([-1.0, 1.0], (k, n))
    _, res, _ = check_against_oracle(g, h, A, B, mode="fixed_guarded", max_bits=55)
    assert (res.fallback, res.esc, res.required_bits, res.slices_used) == (0, 1, 54, 7)
    A[7, 1:] *= 0.5            # one dot product whose best term sits one bit below eA + eB
    B[0, 9] *= 0.5
    B[2:, 9] *= 0.5
    _, res, _ = check_against_oracle(g, h, A, B, mode="fixed_guarded", max_bits=55, bound=False)
    assert (res.fallback, res.reason, res.esc, res.required_bits) == (1, oz.REASON_BITS, 2, 55)
    _, res, _ = check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200)
    assert (res.fallback, res.slices_used) == (0, 8)


def test_grading_test2_guardrails(lib):
    g, h = lib
    A, B, x = wl.grading_test2(96, 40, seed=2)
    _, res, _ = check_against_oracle(g, h, A, B, mode="fixed_guarded", max_bits=55, bound=False)
    assert (res.fallback, res.reason, res.esc) == (1, oz.REASON_BITS, 81)
    _, res, _ = check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200)
    assert res.fallback == 0 and res.slices_used == oz.slices_dynamic(53, 81)


def test_grade_a_sweep_uniform01(lib):
    # Aspect A2 of section "Numerical Accuracy": U(0,1) squares, maximum and average componentwise
    # relative error |fl(AB) - AB| / (|A||B|) against n, measured against the exact reference (not
    # against any product of the library) on 1000 sampled entries per matrix.  Grade A: the maximum
    # stays below f(n)*eps with f at most linear in n (here f = n, eps = 2^-53).  Observed shape, also
    # asserted: the emulated results (dynamic and forced to 55 bits) carry a few eps whatever n is,
    # the native FP64 GEMM's average error grows like sqrt(n).
    g, h = lib
    eps = 2.0 ** -53
    stats = {}
    for nn in (256, 1024):
        for seed in (1, 2):
            A, B = wl.uniform_01(nn, nn, nn, seed=100 * nn + seed)
            pick = np.random.default_rng(seed).choice(nn * nn, 1000, replace=False)
            idx = [(int(t // nn), int(t % nn)) for t in pick]
            exact = ex.exact_entries(A, B, idx)
            den = ex.bound_denominator(A, B, idx)
            for name, opt in (("dynamic", dict(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0)),
                              ("forced55", dict(mode=g.OZ_FORCED_GUARDED, max_bits=55)),
                              ("native", dict(mode=g.OZ_NATIVE))):
                got, _, res = run_gpu(g, h, A, B, **opt)
                rel = np.abs(np.array([got[i, j] for i, j in idx]) - exact) / den / eps
                assert rel.max() <= nn, (name, nn, seed, rel.max())
                stats.setdefault((name, nn), []).append((rel.max(), rel.mean()))
                if name != "native":
                    assert res.fallback == 0
    mx = {key: max(v[0] for v in val) for key, val in stats.items()}
    av = {key: float(np.mean([v[1] for v in val])) for key, val in stats.items()}
    for name in ("dynamic", "forced55"):
        assert mx[(name, 256)] <= 4.0 and mx[(name, 1024)] <= 4.0, mx       # flat in n, a few eps
    assert av[("dynamic", 1024)] <= av[("forced55", 1024)] <= av[("native", 1024)], av
    trend = av[("native", 1024)] / av[("native", 256)]
    assert 1.3 <= trend <= 3.0, trend                                        # sqrt(4) = 2, not 4


def test_adversarial_wide_span_falls_back(lib):
    g, h = lib
    A, B = wl.wide_span(260, 300, 130, seed=7)
    got, res, _ = check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200, bound=False)
    assert (res.fallback, res.reason) == (1, oz.REASON_BITS) and res.esc > 600
    idx = [(i, j) for i in range(0, 260, 37) for j in range(0, 130, 17)]
    exact = ex.exact_entries(A, B, idx)
    den = ex.bound_denominator(A, B, idx)
    assert ex.gradeA_ratio(np.array([got[i, j] for i, j in idx]), exact, den, 300) <= 1.0


def test_adversarial_inf_nan_falls_back(lib):
    g, h = lib
    A0, B0 = wl.lognormal_spread(150, 260, 140, 0.5, seed=8)
    A, B = wl.plant_inf_nan(A0, B0, seed=8)
    got, res, _ = check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200, bound=False)
    assert (res.fallback, res.reason, res.infnan) == (1, oz.REASON_INFNAN, 1)
    with np.errstate(all="ignore"):
        ref = A @ B
    np.testing.assert_array_equal(np.isnan(got), np.isnan(ref))
    np.testing.assert_array_equal(np.isinf(got), np.isinf(ref))
    fin = np.isfinite(ref)
    assert np.allclose(got[fin], ref[fin], rtol=1e-10, atol=1e-10)
    # forced mode also yields to Inf/NaN
    _, res, _ = check_against_oracle(g, h, A, B, mode="forced", max_bits=55, bound=False)
    assert res.reason == oz.REASON_INFNAN


def test_adversarial_rank1_cancellation(lib):
    g, h = lib
    A, B = wl.rank1_cancel(200, 300, 100, seed=9)
    _, res, _ = check_against_oracle(g, h, A, B, mode="dynamic", max_bits=200)
    assert res.fallback == 0 and res.slices_used >= 8


def test_row_scaling_invariance(lib):
    # config 4's structure: row i of A times 2^(i mod 40) leaves the digits unchanged and scales C exactly
    g, h = lib
    A, B, A0 = wl.row_scaled(128, 512, 64, seed=6)
    got, _, tr = check_against_oracle(g, h, A, B, mode="forced", max_bits=55)
    got0, _, tr0 = check_against_oracle(g, h, A0, B, mode="forced", max_bits=55)
    np.testing.assert_array_equal(tr.As, tr0.As)
    scale = np.ldexp(1.0, (np.arange(128) % 40).astype(np.int32))[:, None]
    np.testing.assert_array_equal(got, got0 * scale)


def test_emergent_infinity(lib):
    g, h = lib
    A = np.full((3, 8), 1.5e200)
    B = np.full((8, 3), 1.2e200)
    B[:, 1] *= -1
    got, res, _ = check_against_oracle(g, h, A, B, mode="forced", max_bits=55, bound=False)
    assert np.all(got[:, 0] == np.inf) and np.all(got[:, 1] == -np.inf)


def test_degenerate_sizes(lib):
    g, h = lib
    Cin = np.arange(12.0).reshape(3, 4)
    A, B = np.ones((3, 5)), np.ones((5, 4))
    got, _, res = run_gpu(g, h, np.zeros((3, 0)), np.zeros((0, 4)), 1.0, 2.0, Cin, mode=g.OZ_DYNAMIC)
    np.testing.assert_array_equal(got, 2 * Cin)
    got, _, res = run_gpu(g, h, A, B, 0.0, 0.0, Cin, mode=g.OZ_DYNAMIC)
    np.testing.assert_array_equal(got, np.zeros((3, 4)))
    assert (res.fallback, res.slices_used, res.esc) == (0, 0, -1)
    got, _, _ = run_gpu(g, h, np.ones((0, 5)), B, mode=g.OZ_DYNAMIC)      # m == 0: nothing happens
    assert got.shape == (0, 4)
    got, _, _ = run_gpu(g, h, np.full((1, 1), 3.0), np.full((1, 1), -2.0), mode=g.OZ_FORCED_GUARDED, max_bits=55)
    assert got[0, 0] == -6.0


def test_heuristic_sends_small_problems_native(lib):
    g, h = lib
    A, B = wl.uniform_pm1(48, 48, 48, seed=30)
    got, _, res = run_gpu(g, h, A, B, mode=g.OZ_DYNAMIC, max_bits=200, heuristic=1)
    # no slice count this shape could get beats the native GEMM: native without a scan
    v = oz.emulated_dgemm(A, B, mode=oz.MODE_DYNAMIC, max_bits=200, heuristic=oz.HeuristicModel()).verdict
    assert (v.fallback, v.reason, v.esc) == (1, oz.REASON_HEURISTIC, -1)
    assert (res.fallback, res.reason, res.slices_used, res.esc, res.required_bits, res.infnan) == \
           (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits, v.infnan)
    assert np.allclose(got, A @ B, rtol=0, atol=48 * 2.0 ** -53 * 48)


def test_heuristic_after_the_esc(lib):
    # a shape where 7 slices would pay but the ESC asks for more: scanned, then native by the heuristic
    g, h = lib
    A, B = wl.lognormal_spread(4096, 4096, 4096, 1.0, seed=31)
    m = 4096
    opts = g.make_opts(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=1)
    gm = g.Gemm(h, m, m, m, opts)
    dA, dB = g.to_colmajor(A), g.to_colmajor(B)
    dC = torch.empty((m, m), dtype=torch.float64, device="cuda")
    gm.run(dA, m, dB, m, dC, m)
    torch.cuda.synchronize()
    res = gm.result()
    assert not oz.shape_only_fallback(oz.MODE_DYNAMIC, 53, m, m, m, oz.HeuristicModel())
    v = oz.verdict(oz.MODE_DYNAMIC, 53, 200, 0, False, res.esc, m, m, m, oz.HeuristicModel())
    assert res.esc > 1
    assert (res.fallback, res.reason, res.slices_used, res.required_bits) == \
           (v.fallback, v.reason, v.slices_used, v.required_bits)
    assert (v.fallback, v.reason) == (1, oz.REASON_HEURISTIC)


# 64-tiles: ragged and interior; 128-tiles (at least 256 of them): ragged and interior
@pytest.mark.parametrize("shape", [(200, 150, 333), (256, 384, 512), (2100, 2050, 50), (2048, 2048, 64), (33, 17, 9),
                                   (300, 260, 31), (2049, 2177, 129), (129, 4097, 16),
                                   # few tiles and a long k: the k range is split over several workgroups per tile
                                   (256, 300, 20000), (1000, 900, 4100), (1024, 1024, 8192), (128, 128, 1024)])
@pytest.mark.parametrize("ta,tb", [("N", "N"), ("T", "N"), ("N", "T"), ("T", "T")])
def test_native_fp64_gemm(lib, ta, tb, shape):
    g, h = lib
    m, n, k = shape
    A, B, Cin = wl.lognormal_spread(m, k, n, 0.5, seed=40, with_c=True)
    got, _, res = run_gpu(g, h, A, B, 1.5, 0.5, Cin, ta, tb, pad=2 if m % 128 else 0, mode=g.OZ_NATIVE)
    assert (res.fallback, res.reason) == (1, oz.REASON_NATIVE)
    idx = [(i, j) for i in range(0, m, 13 if m < 1000 else 131) for j in range(0, n, 11 if n < 1000 else 127)]
    idx += [(m - 1, n - 1), (0, n - 1), (m - 1, 0)]
    exact = ex.exact_entries(A, B, idx, 1.5, 0.5, Cin)
    den = ex.bound_denominator(A, B, idx, 1.5, 0.5, Cin)
    assert ex.gradeA_ratio(np.array([got[i, j] for i, j in idx]), exact, den, k) <= 1.0
    # every entry (edge tiles included) against the host product: both sides are within k*2^-53 of the exact value
    full = 1.5 * (A @ B) + 0.5 * Cin
    slack = 2.0 * (k + 2) * 2.0 ** -53 * (1.5 * (np.abs(A) @ np.abs(B)) + 0.5 * np.abs(Cin))
    assert np.all(np.abs(got - full) <= slack)


@pytest.mark.parametrize("seed", range(12))
def test_randomized_native_shapes(lib, seed):
    # the FP64 fallback over drawn shapes (small with a long k, tall, wide, short k), transposes, scalars and
    # leading dimensions, reached both as OZ_NATIVE (small workspace) and through the guard on an Inf in A
    # (workspace of the default mode, so skinny products split k): every finite entry of the host product is
    # matched inside the bound, every other entry is Inf or NaN
    g, h = lib
    rng = np.random.default_rng(31000 + seed)
    kind = seed % 4
    if kind == 0:
        m, n, k = int(rng.integers(1, 600)), int(rng.integers(1, 600)), int(rng.integers(1, 9000))
    elif kind == 1:
        m, n, k = int(rng.integers(1, 3000)), int(rng.integers(1, 300)), int(rng.integers(500, 5000))
    elif kind == 2:
        m, n, k = int(rng.integers(1, 300)), int(rng.integers(1, 3000)), int(rng.integers(500, 5000))
    else:
        m, n, k = int(rng.integers(100, 2200)), int(rng.integers(100, 2200)), int(rng.integers(1, 700))
    A, B, Cin = rng.standard_normal((m, k)), rng.standard_normal((k, n)), rng.standard_normal((m, n))
    alpha, beta = float(rng.choice([1.0, -1.5, 0.3])), float(rng.choice([0.0, 1.0, 0.5]))
    ta, tb = str(rng.choice(["N", "T"])), str(rng.choice(["N", "T"]))
    guarded = bool(seed & 4)
    opt = dict(mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200, heuristic=0) if guarded else dict(mode=g.OZ_NATIVE)
    if guarded:
        A[int(rng.integers(m)), int(rng.integers(k))] = np.inf
    got, _, res = run_gpu(g, h, A, B, alpha, beta, Cin if beta else None, ta, tb, pad=int(rng.integers(0, 3)), **opt)
    assert (res.fallback, res.reason) == (1, oz.REASON_INFNAN if guarded else oz.REASON_NATIVE)
    with np.errstate(all="ignore"):
        want = alpha * (A @ B) + (beta * Cin if beta else 0.0)
        slack = 2.0 * (k + 2) * 2.0 ** -53 * (abs(alpha) * (np.abs(A) @ np.abs(B)) + abs(beta) * np.abs(Cin))
        fin = np.isfinite(want) & np.isfinite(slack)
    assert np.all(np.abs(got[fin] - want[fin]) <= slack[fin])
    assert not np.isfinite(got[~fin]).any()


@pytest.mark.parametrize("shape", [(300, 260, 9000), (2304, 2200, 1100)])
def test_native_k_split_is_reproducible_and_serves_the_guarded_call(lib, shape):
    # a product falls back on a NaN: the native GEMM splits k over several workgroups per tile (few tiles and a
    # long k; or 18 x 18 tiles, 1.27 per CU, where two parts per tile shorten the last round) and adds the parts
    # in a fixed order, so the result is the same on every run and equals the host product within the bound
    # wherever the NaN does not reach
    g, h = lib
    m, n, k = shape
    A, B = wl.lognormal_spread(m, k, n, 0.5, seed=44)
    A[17, k // 2] = np.nan
    outs = []
    for _ in range(2):
        got, _, res = run_gpu(g, h, A, B, 1.0, 0.0, None, "N", "N", mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200,
                              heuristic=0)
        assert (res.fallback, res.reason) == (1, oz.REASON_INFNAN)
        outs.append(got)
    assert np.array_equal(np.isnan(outs[0]), np.isnan(outs[1]))
    assert np.array_equal(np.nan_to_num(outs[0]), np.nan_to_num(outs[1]))
    assert np.all(np.isnan(outs[0][17, :])) and not np.isnan(np.delete(outs[0], 17, axis=0)).any()
    rows = np.array([r for r in range(m) if r != 17])
    full = A[rows] @ B
    slack = 2.0 * (k + 2) * 2.0 ** -53 * (np.abs(A[rows]) @ np.abs(B))
    assert np.all(np.abs(outs[0][rows] - full) <= slack)


@pytest.mark.parametrize("seed", range(16))
def test_randomized_configurations(lib, seed):
    # shapes, modes, transposes, scalars, leading dimensions, exponent spreads and block lengths drawn
    # from a seeded generator; everything the oracle defines must match bit for bit
    g, h = lib
    rng = np.random.default_rng(1000 + seed)
    m, n, k = int(rng.integers(1, 260)), int(rng.integers(1, 300)), int(rng.integers(1, 500))
    phi = float(rng.choice([0.0, 0.3, 1.0, 2.0]))
    A, B, Cin = wl.lognormal_spread(m, k, n, phi, seed=2000 + seed, with_c=True)
    if rng.random() < 0.3:                               # sprinkle zeros, a zero row and a zero column
        A[rng.random(A.shape) < 0.05] = 0.0
        A[int(rng.integers(m)), :] = 0.0
        B[:, int(rng.integers(n))] = 0.0
    mode = str(rng.choice(["dynamic", "forced", "fixed_guarded", "unguarded"]))
    alpha = float(rng.choice([1.0, -1.0, 0.75, 3.0]))
    beta = float(rng.choice([0.0, 1.0, -0.5]))
    ta, tb = str(rng.choice(["N", "T"])), str(rng.choice(["N", "T"]))
    max_bits = 200 if mode == "dynamic" else int(rng.choice([39, 55, 63]))
    check_against_oracle(g, h, A, B, alpha, beta, Cin if beta != 0.0 else None, mode=mode, max_bits=max_bits,
                         esc_block=int(rng.choice([0, 16, 32, 128])), transa=ta, transb=tb,
                         pad=int(rng.integers(0, 4)), bound=(mode == "dynamic"))


@pytest.mark.parametrize("seed", range(8))
def test_randomized_configurations_multi_tile(lib, seed):
    # the same draw over shapes that span several 256 x 256 blocks of C, a k split or several rounds, wider
    # exponent spreads, operands scaled towards the ends of the FP64 range, other target precisions
    g, h = lib
    rng = np.random.default_rng(5000 + seed)
    m, n, k = int(rng.integers(1, 900)), int(rng.integers(1, 900)), int(rng.integers(1, 1500))
    phi = float(rng.choice([0.0, 0.3, 1.0, 2.0, 4.0]))
    A, B, Cin = wl.lognormal_spread(m, k, n, phi, seed=7000 + seed, with_c=True)
    if rng.random() < 0.3:
        A[rng.random(A.shape) < 0.05] = 0.0
        A[int(rng.integers(m)), :] = 0.0
        B[:, int(rng.integers(n))] = 0.0
    if rng.random() < 0.25:
        A *= 2.0 ** float(rng.integers(-1000, 900))
    mode = str(rng.choice(["dynamic", "forced", "fixed_guarded", "unguarded"]))
    alpha = float(rng.choice([1.0, -1.0, 0.75, 3.0, 1.1]))
    beta = float(rng.choice([0.0, 1.0, -0.5, 0.3]))
    ta, tb = str(rng.choice(["N", "T"])), str(rng.choice(["N", "T"]))
    max_bits = 200 if mode == "dynamic" else int(rng.choice([23, 39, 55, 63, 87]))
    tbits = int(rng.choice([53, 53, 40, 64])) if mode == "dynamic" else 53
    check_against_oracle(g, h, A, B, alpha, beta, Cin if beta != 0.0 else None, mode=mode, max_bits=max_bits,
                         target_bits=tbits, esc_block=int(rng.choice([0, 16, 32, 128])), transa=ta, transb=tb,
                         pad=int(rng.integers(0, 4)), bound=(mode == "dynamic" and tbits >= 53))


@pytest.mark.parametrize("seed", range(8))
def test_randomized_per_tile_slice_counts(lib, seed):
    # per-block slice counts on drawn shapes and inputs (a band of difficult rows, i.i.d. spreads, zeros in both
    # operands), with and without the cost model: record, per-block counts and C bit for bit
    g, h = lib
    rng = np.random.default_rng(9000 + seed)
    m, n, k = int(rng.integers(1, 1100)), int(rng.integers(1, 1100)), int(rng.integers(1, 900))
    kind = int(rng.integers(3))
    if kind == 0 and m > 40:
        r0 = int(rng.integers(0, m - 20))
        A, B = wl.wide_rows(m, k, n, seed=seed, row_lo=r0, row_hi=r0 + int(rng.integers(1, 20)),
                            spread=int(rng.integers(8, 60)))
    else:
        A, B = wl.lognormal_spread(m, k, n, float(rng.choice([0.3, 1.0, 3.0])), seed=seed)
        if kind == 2:
            A[rng.random(A.shape) < 0.1] = 0.0
            B[rng.random(B.shape) < 0.1] = 0.0
    Cin = rng.standard_normal((m, n))
    alpha, beta = float(rng.choice([1.0, 1.5, -0.7])), float(rng.choice([0.0, 0.5]))
    ta, tb = str(rng.choice(["N", "T"])), str(rng.choice(["N", "T"]))
    tbits = int(rng.choice([53, 53, 45, 61]))
    hz = int(rng.integers(2))
    got, gm, res = run_gpu(g, h, A, B, alpha, beta, Cin if beta else None, ta, tb, pad=int(rng.integers(0, 3)),
                           mode=g.OZ_DYNAMIC, target_bits=tbits, max_bits=200, heuristic=hz, tile_slices=1)
    tr = oz.emulated_dgemm(A, B, alpha, beta, Cin if beta else None, mode=oz.MODE_DYNAMIC, target_bits=tbits,
                           max_bits=200, per_tile=True, heuristic=oz.HeuristicModel() if hz else None)
    v = tr.verdict
    assert (res.fallback, res.reason, res.slices_used, res.esc, res.required_bits, res.infnan, res.slices_min,
            res.pair_tiles) == (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits, v.infnan, v.slices_min,
                                v.pair_tiles)
    if not v.fallback:
        np.testing.assert_array_equal(gm.tile_slice_counts(), tr.S_tile)
        np.testing.assert_array_equal(got, tr.C)


@pytest.mark.parametrize("ta,tb,seed", [("N", "N", 0), ("T", "N", 1), ("N", "T", 2), ("T", "T", 3)])
def test_per_tile_slice_counts(lib, ta, tb, seed):
    # OZ_DYNAMIC with tile_slices: a band of difficult rows makes the blocks of C it crosses need more
    # slices than the rest.  Record (with the pair count), the per-block slice counts, every
    # anti-diagonal a block walked, and C must equal the oracle's; the bound must hold everywhere.
    g, h = lib
    m, n, k = 600, 700, 300 + 40 * seed
    row0 = [10, 300, 560, 250][seed]
    A, B = wl.wide_rows(m, k, n, seed=90 + seed, row_lo=row0, row_hi=row0 + 12, spread=20 + 4 * seed)
    Cin = np.random.default_rng(seed).standard_normal((m, n))
    got, gm, res = run_gpu(g, h, A, B, 1.5, 0.5, Cin, ta, tb, pad=seed, mode=g.OZ_DYNAMIC, target_bits=53,
                           max_bits=200, heuristic=0, tile_slices=1)
    tr = oz.emulated_dgemm(A, B, 1.5, 0.5, Cin, mode=oz.MODE_DYNAMIC, target_bits=53, max_bits=200, per_tile=True)
    v = tr.verdict
    assert (res.fallback, res.reason, res.slices_used, res.esc, res.required_bits, res.infnan, res.slices_min,
            res.pair_tiles) == (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits, v.infnan, v.slices_min,
                                v.pair_tiles)
    whole = oz.verdict(oz.MODE_DYNAMIC, 53, 200, 0, False, v.esc, m, n, k)
    assert v.slices_min < v.slices_used and v.pair_tiles < whole.pair_tiles       # fewer pair products than one count for all
    np.testing.assert_array_equal(gm.tile_slice_counts(), tr.S_tile)
    S = v.slices_used
    As, Bs = gm.slices(S)
    np.testing.assert_array_equal(As, tr.As)
    np.testing.assert_array_equal(Bs, tr.Bs)
    gT, glo = gm.digits(S, tr.P.shape[0])
    for ti in range(tr.S_tile.shape[0]):
        for tj in range(tr.S_tile.shape[1]):
            r, c, St = slice(256 * ti, 256 * ti + 256), slice(256 * tj, 256 * tj + 256), int(tr.S_tile[ti, tj])
            T0, lo = oz.normalised_digits(tr.P[:, :St, r, c])          # the block's own anti-diagonals, aggregated
            np.testing.assert_array_equal(gT[:, r, c], T0)
            np.testing.assert_array_equal(glo[:, :St - 1, r, c], lo)
    np.testing.assert_array_equal(got, tr.C)
    pick = np.random.default_rng(seed).choice(m * n, 3000, replace=False)
    idx = [(int(t // n), int(t % n)) for t in pick] + [(i, j) for i in range(row0, row0 + 12) for j in range(0, n, 9)]
    exact = ex.exact_entries(A, B, idx, 1.5, 0.5, Cin)
    den = ex.bound_denominator(A, B, idx, 1.5, 0.5, Cin)
    assert ex.gradeA_ratio(np.array([got[i, j] for i, j in idx]), exact, den, k) <= 1.0


@pytest.mark.parametrize("m,n", [(4096, 4096), (4352, 4100)])
def test_per_tile_counts_with_the_tiles_dealt_by_slice_count(lib, m, n):
    # 16 x 16 blocks of C (one full round of the slice GEMM) or 17 x 17 (a full round and a k-split launch for
    # the 33 blocks left over): the blocks are sorted by slice count and dealt to the XCDs in turn.  The difficult
    # dot products lie in two block columns; whatever order the blocks run in, record, per-block counts and
    # every entry of C are the oracle's
    g, h = lib
    k = 192
    A0, B0 = wl.wide_rows(n, k, m, seed=13, row_lo=1000, row_hi=1040, spread=20)
    A, B = np.ascontiguousarray(B0.T), np.ascontiguousarray(A0.T)          # hard columns of C instead of hard rows
    got, gm, res = run_gpu(g, h, A, B, 1.0, 0.0, None, "N", "N", mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200,
                           heuristic=0, tile_slices=1)
    tr = oz.emulated_dgemm(A, B, 1.0, 0.0, None, mode=oz.MODE_DYNAMIC, target_bits=53, max_bits=200, per_tile=True)
    v = tr.verdict
    assert (res.fallback, res.reason, res.slices_used, res.esc, res.required_bits, res.infnan, res.slices_min,
            res.pair_tiles) == (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits, v.infnan, v.slices_min,
                                v.pair_tiles)
    assert v.slices_min < v.slices_used
    np.testing.assert_array_equal(gm.tile_slice_counts(), tr.S_tile)
    nti, ntj = tr.S_tile.shape
    heavy = np.argwhere(tr.S_tile == v.slices_used)
    assert set(heavy[:, 1].tolist()) == {3, 4} and len(heavy) == 2 * nti       # two block columns
    np.testing.assert_array_equal(got, tr.C)
    # the order table is a permutation of the blocks, and the first round of the first XCD (positions 0..31: the
    # sorted sequence is dealt in groups of 32, group g to XCD g % 8) holds heavy blocks only
    order = gm.tile_order()
    assert sorted(order.tolist()) == list(range(nti * ntj))

    def block_column(lin):      # block order of the GEMM: panels of 8 block columns, inside a panel row by row
        panel = lin // (8 * nti)
        width = min(8, ntj - panel * 8)
        return panel * 8 + (lin - panel * 8 * nti) % width
    assert {block_column(int(t)) for t in order[:32]} <= {3, 4}
    # the blocks left to the k-split launch (behind the full round) are among the lightest
    if nti * ntj > 256:
        S_of = lambda lin: tr.S_tile[(lin - (lin // (8 * nti)) * 8 * nti) // min(8, ntj - (lin // (8 * nti)) * 8), block_column(lin)]
        assert all(S_of(int(t)) == v.slices_min for t in order[256:])


def test_per_tile_cost_model_keeps_a_localised_hard_region_emulated(lib):
    # With one slice count for all of C the cost model sends this input to the native GEMM (the worst
    # block's count applied everywhere is too slow); with per-block counts the mean pair count decides,
    # and only the band pays for its bits.  The constants are set so that the shape itself is in range.
    g, h = lib
    m = n = 1536
    k = 512
    A, B = wl.wide_rows(m, k, n, seed=95, row_lo=700, row_hi=720, spread=60)
    hm = oz.HeuristicModel(int8_ops_per_ns=2650000, fp64_flops_per_ns=30000, bytes_per_ns=40000, fixed_ns=0)
    h2 = g.Handle(0)
    try:
        h2.set_heuristic(hm.int8_ops_per_ns, hm.fp64_flops_per_ns, hm.bytes_per_ns, hm.fixed_ns)
        out = {}
        for tiles in (0, 1):
            got, gm, res = run_gpu(g, h2, A, B, mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200, heuristic=1,
                                   tile_slices=tiles)
            tr = oz.emulated_dgemm(A, B, mode=oz.MODE_DYNAMIC, target_bits=53, max_bits=200, heuristic=hm,
                                   per_tile=bool(tiles))
            v = tr.verdict
            assert (res.fallback, res.reason, res.slices_used, res.esc, res.required_bits, res.slices_min,
                    res.pair_tiles) == (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits, v.slices_min,
                                        v.pair_tiles)
            if not v.fallback:
                np.testing.assert_array_equal(got, tr.C)
            out[tiles] = (v.fallback, v.reason)
        assert out[0] == (1, oz.REASON_HEURISTIC) and out[1] == (0, oz.REASON_NONE), out
    finally:
        h2.close()


def test_blocked_qr_through_oz_dgemm(lib):
    # Blocked Householder QR (section "Application-Level Integration") with the three products of every
    # trailing update going through oz_dgemm.  R is unique up to the signs of its rows, and LAPACK's and
    # the vendor solver's Householder conventions agree, so R is compared with a reference factorisation
    # (numpy / LAPACK on the host) column by column: |R - R_ref|_ij <= c n 2^-53 ||A(:, j)||_2.  The
    # emulated runs must be as close to the reference as the run on the native FP64 GEMM.
    g, h = lib
    from paper_2511_13778_amd.qr import blocked_qr
    n, b = 1024, 128
    A = np.random.default_rng(77).standard_normal((n, n))
    R_ref = np.linalg.qr(A, mode="r")
    colnorm = np.linalg.norm(A, axis=0)
    tol = 64.0 * n * 2.0 ** -53
    errs = {}
    for name, opts in (("native", g.make_opts(mode=g.OZ_NATIVE)),
                       ("dynamic", g.make_opts(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0, tile_slices=1)),
                       ("shipped", g.default_opts())):
        At = g.to_colmajor(A)
        tau, rep = blocked_qr(h, At, b, opts)
        R = np.triu(g.from_colmajor(At))
        sign = np.sign(np.diag(R)) * np.sign(np.diag(R_ref))
        err = np.abs(R * sign[:, None] - R_ref) / colnorm[None, :]
        errs[name] = float(err.max())
        assert errs[name] <= tol, (name, errs[name], tol)
        assert rep.panels == n // b and len(rep.records) == 3 * (n // b - 1)
        hist = rep.histogram()
        if name == "native":
            assert hist == {"native:forced": len(rep.records)}
        if name == "dynamic":          # heuristic off: every product emulated, slice counts from the ESC
            assert all(r.fallback == 0 and r.slices_used >= 7 and r.esc >= 1 for _, _, _, r in rep.records), hist
            # each call's verdict is what the oracle derives from the ESC the device reported
            for mm, nn, kk, r in rep.records:
                assert r.slices_used == oz.slices_dynamic(53, r.esc) and r.slices_min <= r.slices_used
        if name == "shipped":          # at this size the cost model sends every product to the native GEMM
            assert all(r.fallback == 1 and r.reason == oz.REASON_HEURISTIC for _, _, _, r in rep.records), hist
    assert errs["dynamic"] <= 4.0 * errs["native"] + 1e-16, errs


def test_native_gemm_with_a_very_large_leading_dimension(lib):
    # operands cut out of a huge parent matrix: 15 leading dimensions no longer fit a 32-bit byte offset,
    # so the FP64 kernel must take its 64-bit indexing path (interior tile sizes on purpose)
    g, h = lib
    m, n, k = 128, 128, 32
    ld = 36_000_000
    rng = np.random.default_rng(12)
    A, B = rng.standard_normal((m, k)), rng.standard_normal((k, n))
    dA = torch.zeros(k * ld, dtype=torch.float64, device="cuda")           # column-major m x k, lda = ld
    dA.view(k, ld)[:, :m] = torch.from_numpy(np.ascontiguousarray(A.T)).cuda()
    dBt = torch.zeros(k * ld, dtype=torch.float64, device="cuda")          # B^T stored column-major n x k, ldb = ld
    dBt.view(k, ld)[:, :n] = torch.from_numpy(np.ascontiguousarray(B)).cuda()
    dC = torch.zeros((n, m), dtype=torch.float64, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    h.native_dgemm(st, "N", "T", m, n, k, 1.0, dA.data_ptr(), ld, dBt.data_ptr(), ld, 0.0, dC.data_ptr(), m)
    torch.cuda.synchronize()
    got = g.from_colmajor(dC)
    idx = [(i, j) for i in range(0, m, 9) for j in range(0, n, 7)]
    ratio = ex.gradeA_ratio(np.array([got[i, j] for i, j in idx]), ex.exact_entries(A, B, idx),
                            ex.bound_denominator(A, B, idx), k)
    assert ratio <= 1.0, ratio


def test_concurrent_slice_gemms_share_the_chip(lib):
    # Two problems with more tiles than the chip runs at a time (324 > 256), in two lanes of a batched
    # call: their slice GEMMs run concurrently, so the workgroups a tile round waits for may never
    # arrive.  The waits are bounded and only serve cache locality: the results must equal the serial ones.
    g, h = lib
    m = n = 4608
    k = 512
    nb = 2
    mats = [wl.lognormal_spread(m, k, n, 0.5, seed=130 + b) for b in range(nb)]
    opts = g.make_opts(mode=g.OZ_FORCED_GUARDED, max_bits=55)
    one = (h.workspace_bytes("N", "N", m, n, k, opts) + 255) // 256 * 256
    dA = torch.from_numpy(np.stack([a.T.copy() for a, _ in mats])).cuda()
    dB = torch.from_numpy(np.stack([b_.T.copy() for _, b_ in mats])).cuda()
    st = torch.cuda.current_stream().cuda_stream
    outs = []
    for lanes in (1, 2):
        ws = torch.empty(one * lanes, dtype=torch.uint8, device="cuda")
        dC = torch.full((nb, n, m), float("nan"), dtype=torch.float64, device="cuda")
        recs = torch.zeros((nb, g.RESULT_INT32_WORDS), dtype=torch.int32, device="cuda")
        h.dgemm_strided_batched(st, "N", "N", m, n, k, 1.0, dA.data_ptr(), m, m * k, dB.data_ptr(), k, k * n, 0.0,
                                dC.data_ptr(), m, m * n, nb, opts, ws.data_ptr(), one * lanes, recs.data_ptr())
        torch.cuda.synchronize()
        outs.append(dC)
        assert all(g.result_from_words(r).slices_used == 7 for r in recs.cpu().tolist())
    assert torch.equal(outs[0], outs[1])
    # and the serial result is the oracle's, on sampled rows and columns of the first problem
    A, B = mats[0]
    I = np.array([0, 255, 256, 2000, 4607])
    J = np.array([1, 300, 4351, 4352, 4606])
    eA, eB = oz.row_exponents(A), oz.col_exponents(B)
    P = oz.slice_products(oz.slice_rows(A[I], eA[I], 7), oz.slice_rows(np.ascontiguousarray(B[:, J].T), eB[J], 7))
    want = oz.recompose(P, eA[I], eB[J])
    got = outs[1][0].index_select(0, torch.as_tensor(J, device="cuda")).index_select(1, torch.as_tensor(I, device="cuda"))
    np.testing.assert_array_equal(got.cpu().numpy().T, want)


@pytest.mark.parametrize("ta,tb,beta", [("N", "N", 0.0), ("T", "N", complex(0.5, 2.0)), ("N", "C", complex(-1.0, 0.25)),
                                        ("C", "T", 0.0)])
def test_zgemm_4m(lib, ta, tb, beta):
    # complex product by the 4M method: four real products through the emulated DGEMM (each with its own
    # record), combined in a fixed order: bit-identical to the oracle's, and inside the componentwise bound
    # of the exact complex product on sampled entries
    g, h = lib
    rng = np.random.default_rng(hash((ta, tb)) % 1000)
    m, n, k = 150, 270, 333
    cplx = lambda shape: (rng.standard_normal(shape) + 1j * rng.standard_normal(shape)) * np.exp2(rng.integers(-4, 5, shape))
    A, B, Cin = cplx((m, k)), cplx((k, n)), cplx((m, n))
    alpha = complex(1.25, -0.5)
    op = {"N": lambda X: X, "T": lambda X: X.T, "C": lambda X: X.conj().T}
    # stored operands: op(stored) = logical, so stored = op^-1(logical); T and C are their own inverses
    sA, sB = np.ascontiguousarray(op[ta](A)), np.ascontiguousarray(op[tb](B))
    dA = torch.from_numpy(np.ascontiguousarray(sA.T)).cuda()           # column-major storage of the stored matrix
    dB = torch.from_numpy(np.ascontiguousarray(sB.T)).cuda()
    dC = torch.from_numpy(np.ascontiguousarray(Cin.T)).cuda() if beta != 0.0 else \
        torch.full((n, m), complex(float("nan"), float("nan")), dtype=torch.complex128, device="cuda")
    opts = g.make_opts(mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200, heuristic=0, tile_slices=0)
    ws_bytes = h.zgemm_workspace_bytes(ta, tb, m, n, k, opts)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    recs = torch.zeros((4, g.RESULT_INT32_WORDS), dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    h.zgemm(st, ta, tb, m, n, k, alpha, dA.data_ptr(), sA.shape[0], dB.data_ptr(), sB.shape[0], beta, dC.data_ptr(), m,
            opts, ws.data_ptr(), ws_bytes, recs.data_ptr())
    torch.cuda.synchronize()
    got = dC.cpu().numpy().T
    want, verdicts = oz.emulated_zgemm(A, B, alpha, beta, Cin, mode=oz.MODE_DYNAMIC, target_bits=53, max_bits=200)
    for r, v in zip(recs.cpu().tolist(), verdicts):
        r = g.result_from_words(r)
        assert (r.fallback, r.reason, r.slices_used, r.esc, r.required_bits) == \
               (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits)
    np.testing.assert_array_equal(got.real, want.real)
    np.testing.assert_array_equal(got.imag, want.imag)
    # exact complex reference on sampled entries (rational arithmetic)
    from fractions import Fraction as F
    absA, absB = np.abs(A.real) + np.abs(A.imag), np.abs(B.real) + np.abs(B.imag)
    b = complex(beta)
    for i, j in [(0, 0), (m - 1, n - 1), (77, 131), (3, 200), (149, 1)]:
        pr = sum(F(float(A[i, l].real)) * F(float(B[l, j].real)) - F(float(A[i, l].imag)) * F(float(B[l, j].imag)) for l in range(k))
        pi = sum(F(float(A[i, l].real)) * F(float(B[l, j].imag)) + F(float(A[i, l].imag)) * F(float(B[l, j].real)) for l in range(k))
        re = F(alpha.real) * pr - F(alpha.imag) * pi
        im = F(alpha.real) * pi + F(alpha.imag) * pr
        den = (abs(alpha.real) + abs(alpha.imag)) * float(absA[i] @ absB[:, j])
        if beta != 0.0:
            re += F(b.real) * F(float(Cin[i, j].real)) - F(b.imag) * F(float(Cin[i, j].imag))
            im += F(b.real) * F(float(Cin[i, j].imag)) + F(b.imag) * F(float(Cin[i, j].real))
            den += (abs(b.real) + abs(b.imag)) * (abs(Cin[i, j].real) + abs(Cin[i, j].imag))
        tol = (k + 4) * 2.0 ** -53 * den
        assert abs(F(float(got[i, j].real)) - re) <= tol and abs(F(float(got[i, j].imag)) - im) <= tol


def test_strided_batched(lib):
    # four problems of one shape in one call: each takes its own decision (slice counts differ, one
    # falls back on a NaN), results and records per problem as from separate oz_dgemm calls
    g, h = lib
    m, n, k, nb = 150, 120, 300, 4
    As, Bs, Cs = [], [], []
    for b, phi in enumerate([0.0, 2.0, 0.5, 1.0]):
        A, B, Cin = wl.lognormal_spread(m, k, n, phi, seed=60 + b, with_c=True)
        As.append(A); Bs.append(B); Cs.append(Cin)
    As[2][7, 11] = np.nan
    opts = g.make_opts(mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200, heuristic=0)
    one = h.workspace_bytes("N", "N", m, n, k, opts)
    one = (one + 255) // 256 * 256
    dA = torch.from_numpy(np.stack([a.T.copy() for a in As])).cuda()     # (nb, k, m): column-major m x k each
    dB = torch.from_numpy(np.stack([b_.T.copy() for b_ in Bs])).cuda()
    st = torch.cuda.current_stream().cuda_stream
    runs = []
    # room for one problem: the batch runs serially on the caller's stream; room for three: three lanes
    # (streams of the handle, forked from and joined to the caller's stream); same results either way
    for lanes in (1, 3):
        ws_bytes = one * lanes
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
        dC = torch.from_numpy(np.stack([c.T.copy() for c in Cs])).cuda()
        recs = torch.zeros((nb, g.RESULT_INT32_WORDS), dtype=torch.int32, device="cuda")
        h.dgemm_strided_batched(st, "N", "N", m, n, k, -1.0, dA.data_ptr(), m, m * k, dB.data_ptr(), k, k * n, 0.5,
                                dC.data_ptr(), m, m * n, nb, opts, ws.data_ptr(), ws_bytes, recs.data_ptr())
        # work enqueued afterwards on the caller's stream is ordered behind every lane
        tail = dC.sum(dim=(1, 2))
        torch.cuda.synchronize()
        runs.append((dC.cpu().numpy(), recs.cpu().numpy(), tail.cpu().numpy()))
    np.testing.assert_array_equal(runs[0][0], runs[1][0])
    np.testing.assert_array_equal(runs[0][1], runs[1][1])
    np.testing.assert_array_equal(runs[0][2], runs[1][2])
    got, recs = runs[1][0], runs[1][1]
    ws_bytes = one
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    dC = torch.from_numpy(np.stack([c.T.copy() for c in Cs])).cuda()
    seen = set()
    for b in range(nb):
        tr = oz.emulated_dgemm(As[b], Bs[b], -1.0, 0.5, Cs[b], mode=oz.MODE_DYNAMIC, target_bits=53, max_bits=200)
        v = tr.verdict
        r = g.result_from_words(recs[b])
        assert (r.fallback, r.reason, r.slices_used, r.esc, r.required_bits, r.infnan, r.slices_min, r.pair_tiles) == \
               (v.fallback, v.reason, v.slices_used, v.esc, v.required_bits, v.infnan, v.slices_min, v.pair_tiles)
        if v.fallback:
            assert np.isnan(got[b].T[7, :]).all()
        else:
            np.testing.assert_array_equal(got[b].T, tr.C)
            seen.add(v.slices_used)
    assert recs[2][0] == 1 and recs[2][1] == oz.REASON_INFNAN and len(seen) >= 2
    # overlapping C blocks are refused before anything runs
    with pytest.raises(g.OzError):
        h.dgemm_strided_batched(st, "N", "N", m, n, k, 1.0, dA.data_ptr(), m, m * k, dB.data_ptr(), k, k * n, 0.0,
                                dC.data_ptr(), m, m * n - 1, nb, opts, ws.data_ptr(), ws_bytes, None)


def test_call_can_be_captured_in_a_graph(lib):
    # the call only enqueues kernels (no allocation, no memset, no synchronisation), so it can be
    # captured; every replay must reproduce the eager result, with eager calls between the replays
    g, h = lib
    n = 300
    A, B = wl.lognormal_spread(n, n, n, 1.0, seed=70)
    dA, dB = g.to_colmajor(A), g.to_colmajor(B)
    dC = torch.zeros((n, n), dtype=torch.float64, device="cuda")
    gm = g.Gemm(h, n, n, n, g.make_opts(mode=g.OZ_DYNAMIC, max_bits=200, heuristic=0))
    gm.run(dA, n, dB, n, dC, n)
    torch.cuda.synchronize()
    ref = dC.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gm.run(dA, n, dB, n, dC, n)                   # warm-up on a side stream, as capture requires
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gm.run(dA, n, dB, n, dC, n)
    for _ in range(3):
        dC.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dC, ref)
        gm.run(dA, n, dB, n, dC, n)
        torch.cuda.synchronize()
        assert torch.equal(dC, ref)
    assert gm.result().fallback == 0
    # the decision is taken on the device, so the same captured graph serves a call that falls back: plant a
    # NaN in A, replay, compare with the eager call on the same operands, then heal A and replay once more
    keep = dA[5, 7].item()
    dA[5, 7] = float("nan")
    dC.fill_(0.0)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    r = gm.result()
    assert (r.fallback, r.reason) == (1, oz.REASON_INFNAN)
    replayed = dC.clone()
    dC.fill_(0.0)
    gm.run(dA, n, dB, n, dC, n)
    torch.cuda.synchronize()
    assert torch.equal(torch.isnan(dC), torch.isnan(replayed)) and torch.isnan(dC).any()
    assert torch.equal(torch.nan_to_num(dC), torch.nan_to_num(replayed))
    dA[5, 7] = keep
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(dC, ref) and gm.result().fallback == 0


def test_argument_errors(lib):
    g, h = lib
    opts = g.make_opts(mode=g.OZ_FORCED_GUARDED, max_bits=55)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    d = torch.zeros(64 * 64, dtype=torch.float64, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    need = h.workspace_bytes("N", "N", 64, 64, 64, opts)
    assert need > 0
    def call(ta="N", tb="N", m=64, n=64, k=64, lda=64, ldb=64, ldc=64, wsb=None, o=opts):
        h.dgemm(st, ta, tb, m, n, k, 1.0, d.data_ptr(), lda, d.data_ptr(), ldb, 0.0, d.data_ptr(), ldc, o,
                ws.data_ptr(), need if wsb is None else wsb)
    for kw, status in (({"ta": "X"}, 1), ({"m": -1}, 1), ({"lda": 63}, 1), ({"ldb": 10}, 1), ({"ldc": 1}, 1),
                       ({"wsb": need - 1}, 2), ({"o": g.make_opts(mode=9)}, 1),
                       ({"o": g.make_opts(esc_block=24)}, 1), ({"o": g.make_opts(max_bits=500)}, 1)):
        with pytest.raises(g.OzError) as e:
            call(**kw)
        assert e.value.status == status
    assert h.workspace_bytes("N", "Q", 64, 64, 64, opts) == 0
    # sizes beyond what the launch grids carry are refused, not launched
    assert h.workspace_bytes("N", "N", 64, 64, (1 << 21) + 1, opts) == 0
    assert h.workspace_bytes("N", "N", (1 << 22) + 1, 64, 64, opts) == 0
    assert h.workspace_bytes("N", "N", 64, 64, 1 << 21, opts) > 0
    torch.cuda.synchronize()
