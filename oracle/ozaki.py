"""CPU oracle for FP64 GEMM emulated with Ozaki scheme I on 8-bit integer slices.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import it.  It shares no code with the HIP library and
never calls it.  Everything here is plain numpy / Python integers, written for legibility:
each function follows one passage of the paper (cited by section) in the paper's order, with
no blocking, fusion or reordering beyond what that passage states.

Notation (paper, section "ESC: Exponent Span Capacity Estimation"):
  A is m x k, B is k x n, C is m x n, all FP64.
  exp(x)  = floor(log2|x|) for finite non-zero x (true exponent, also for denormals).
  eA_i    = max_l exp(a_il)  (row exponent of A),  eB_j = max_l exp(b_lj) (column exponent of B).
  S       = number of 8-bit slices.

Readings of points the paper leaves open (all listed again in the design notes):
  * one headroom bit H=1 in the leading digit so the carry of the unsigned-slice remap can
    never leave the s8 range:  X = floor(a * 2^(8S-2-H-eA)),  |X| < 2^(8S-2);
  * slice pairs (s,t) with s+t <= S-1 are multiplied (S(S+1)/2 products): the count that makes
    7 slices "22 % less compute" than 8 (28/36), section "Unsigned Slice Encoding";
  * in a block minimum a zero counts as -infinity, in a block maximum zeros are ignored; a
    dot product in which every block has an all-zero side needs no bits at all;
  * ESC values are reported clamped to ESC_CAP.

Pins (tests/test_oracle_*.py): the worked encoding example of section "Unsigned Slice
Encoding"; exact reconstruction of floor(a*2^q); brute-force ESC; coarse >= exact; b=1 coarse ==
exact; closed-form ESC of the generalised Test-2 matrices (2b+1); power-of-two scaling
invariance; integer matrices reproduce an int64 matmul exactly; exact rational reference.
Parity unpinned (own choices, only the error bound applies): the run-time heuristic's
cost model, its constants and its shape-only pre-check, the default block length b, the slice
cap, the int32 k-block length, the order of the carry-normalised FP64 recomposition beyond seven
slices (up to seven it is the exact integer rounded once, which is pinned).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from fractions import Fraction

import numpy as np

H = 1                      # headroom bits in the leading digit
ZERO_EXP = -(1 << 20)      # stands for exp(0) = -infinity
NEG_INF_BELOW = -(1 << 19)  # any exponent (or exponent sum) below this is -infinity
ESC_CAP = 4096             # reported ESC is min(ESC, ESC_CAP)
MAX_SLICES = 26            # 200 mantissa bits (section "Numerical Accuracy", aspect A2)
DEFAULT_ESC_BLOCK = 64
TILE = 256                 # edge of the blocks of C that may take their own slice count

MODE_DYNAMIC, MODE_FORCED_GUARDED, MODE_FIXED_GUARDED, MODE_FIXED_UNGUARDED, MODE_NATIVE = range(5)
REASON_NONE, REASON_INFNAN, REASON_BITS, REASON_HEURISTIC, REASON_NATIVE = range(5)


# --------------------------------------------------------------------------------------
# O1  exponents and the Inf/NaN scan  (section "Pre-processing and Safety Checks")
# --------------------------------------------------------------------------------------
def exponents(x: np.ndarray) -> np.ndarray:
    """exp(x) elementwise as int64; zeros (of either sign) give ZERO_EXP.

    frexp writes x = f * 2^p with 0.5 <= |f| < 1, for denormals too, hence exp(x) = p - 1.
    Inf/NaN entries must have been excluded by the caller (see has_inf_nan)."""
    x = np.asarray(x, dtype=np.float64)
    _, p = np.frexp(x)
    e = p.astype(np.int64) - 1
    return np.where(x == 0.0, ZERO_EXP, e)


def has_inf_nan(x: np.ndarray) -> bool:
    """True iff any entry has an all-ones exponent field."""
    return bool(np.any(~np.isfinite(np.asarray(x, dtype=np.float64))))


def row_exponents(A: np.ndarray) -> np.ndarray:
    """eA_i = max_l exp(a_il); an all-zero row gives ZERO_EXP."""
    return exponents(A).max(axis=1)


def col_exponents(B: np.ndarray) -> np.ndarray:
    """eB_j = max_l exp(b_lj); an all-zero column gives ZERO_EXP."""
    return exponents(B).max(axis=0)


# --------------------------------------------------------------------------------------
# O2  exact (non-coarsened) ESC  (section "ESC", the formula for one dot product, maximised
#     over the mn dot products, plus the +1 safety margin)
# --------------------------------------------------------------------------------------
def esc_exact(A: np.ndarray, B: np.ndarray) -> int:
    """max_ij [ exp(x_p) + exp(y_q) - exp(z_r) ] + 1 by brute force (tiny inputs only).

    For the dot product of row i of A with column j of B: exp(x_p) = eA_i, exp(y_q) = eB_j,
    exp(z_r) = max_l (exp(a_il) + exp(b_lj)) over the l whose product is non-zero.  A dot
    product with no non-zero term contributes 0.  Result clamped to ESC_CAP."""
    EA, EB = exponents(A), exponents(B)
    m, k = EA.shape
    n = EB.shape[1]
    best = 0
    for i in range(m):
        for j in range(n):
            zr = None
            for l in range(k):
                if EA[i, l] > NEG_INF_BELOW and EB[l, j] > NEG_INF_BELOW:
                    s = int(EA[i, l] + EB[l, j])
                    zr = s if zr is None else max(zr, s)
            if zr is None:
                continue
            best = max(best, int(EA[i].max()) + int(EB[:, j].max()) - zr)
    return min(best + 1, ESC_CAP)


# --------------------------------------------------------------------------------------
# O3  coarsened ESC  (section "ESC", the paragraph on blocks of length b)
# --------------------------------------------------------------------------------------
def block_minmax(E: np.ndarray, b: int, axis: int):
    """Per length-b block along `axis` (last block may be short): Max exponent over the
    non-zero entries, Min exponent, and two flags: `live` (the block has a non-zero entry, so
    Max exists) and `full` (the block has no zero entry, so Min is finite).
    Returns (Max, Min, live, full) with the blocked axis of length ceil(k/b); Max/Min hold
    ZERO_EXP where they do not exist."""
    E = np.moveaxis(np.asarray(E, dtype=np.int64), axis, -1)
    k = E.shape[-1]
    G = -(-k // b)
    mx = np.empty(E.shape[:-1] + (G,), dtype=np.int64)
    mn = np.empty_like(mx)
    for g in range(G):
        blk = E[..., g * b:min(k, (g + 1) * b)]
        mx[..., g] = blk.max(axis=-1)      # ZERO_EXP is below every real exponent
        mn[..., g] = blk.min(axis=-1)
    live = mx > NEG_INF_BELOW
    full = mn > NEG_INF_BELOW
    return tuple(np.moveaxis(t, -1, axis) for t in (mx, mn, live, full))


def coarse_span(A: np.ndarray, B: np.ndarray, b: int = DEFAULT_ESC_BLOCK) -> np.ndarray:
    """m x n matrix of  eA_i + eB_j - zt_ij  (the coarsened exponent span of every dot product),
    zt_ij = max_g max( Max(xb_g) + Min(yb_g), Min(xb_g) + Max(yb_g) ).

    A zero has exponent -infinity: it never sets a block's Max, and it makes the block's Min
    -infinity, which removes that candidate (the proof that the coarse zt never exceeds the
    true exp(z_r) pairs the entry attaining Max(xb_g) with its partner in yb_g, which must
    therefore be non-zero).  A dot product in which every block has an all-zero side is
    identically zero and has span 0, as in esc_exact.  Any other pair left without a
    candidate is unbounded and gets ESC_CAP."""
    EA, EB = exponents(A), exponents(B)
    eA, eB = EA.max(axis=1), EB.max(axis=0)
    Amax, Amin, Alive, Afull = block_minmax(EA, b, axis=1)          # m x G
    Bmax, Bmin, Blive, Bfull = block_minmax(EB, b, axis=0)          # G x n
    m, G = Amax.shape
    n = Bmax.shape[1]
    zt = np.zeros((m, n), dtype=np.int64)
    have = np.zeros((m, n), dtype=bool)              # zt holds at least one candidate
    dead = np.ones((m, n), dtype=bool)               # every block so far has an all-zero side
    for g in range(G):
        for hi, lo, ok in ((Amax[:, g][:, None], Bmin[g, :][None, :], Alive[:, g][:, None] & Bfull[g, :][None, :]),
                           (Bmax[g, :][None, :], Amin[:, g][:, None], Blive[g, :][None, :] & Afull[:, g][:, None])):
            cand = hi + lo
            zt = np.where(ok & have, np.maximum(zt, cand), np.where(ok, cand, zt))
            have |= ok
        dead &= ~(Alive[:, g][:, None] & Blive[g, :][None, :])
    span = np.where(have, eA[:, None] + eB[None, :] - zt, ESC_CAP)
    return np.where(dead, 0, span)


def esc_coarse(A: np.ndarray, B: np.ndarray, b: int = DEFAULT_ESC_BLOCK) -> int:
    """1 + max_ij of coarse_span, clamped to ESC_CAP: the coarsened ESC of the whole product."""
    span = coarse_span(A, B, b)
    return min(max(int(span.max(initial=0)), 0) + 1, ESC_CAP)


def esc_coarse_tiles(A: np.ndarray, B: np.ndarray, b: int = DEFAULT_ESC_BLOCK, tile: int = 256) -> np.ndarray:
    """ceil(m/tile) x ceil(n/tile) matrix: the coarsened ESC of every tile x tile block of C taken
    on its own, i.e. 1 + the maximum of coarse_span over the dot products of that block only.
    The row and column exponents, and hence the spans, are those of the whole product: a tile's
    rows are still aligned to the maximum of the entire row of A.  (Section "Limitations and
    Future Directions": tighter estimates; the ESC is a per-dot-product quantity, section "ESC",
    and nothing forces one slice count on all of C.)"""
    span = coarse_span(A, B, b)
    m, n = span.shape
    out = np.zeros((-(-m // tile), -(-n // tile)), dtype=np.int64)
    for ti in range(out.shape[0]):
        for tj in range(out.shape[1]):
            blk = span[ti * tile:(ti + 1) * tile, tj * tile:(tj + 1) * tile]
            out[ti, tj] = min(max(int(blk.max(initial=0)), 0) + 1, ESC_CAP)
    return out


# --------------------------------------------------------------------------------------
# O4  slice count and fallback verdict  (sections "Heuristic run time Selection" and
#     "Numerical Accuracy", aspect A1; flowchart of the decision process)
# --------------------------------------------------------------------------------------
def slices_for_bits(bits: int) -> int:
    """Slices that hold `bits` mantissa bits plus the sign: 53 -> 7, 55 -> 7, 63 -> 8."""
    return max(1, -(-(bits + 1) // 8))


def slices_signed_scheme(bits: int) -> int:
    """The encoding the paper improves on: 8 bits in the leading slice, 7 in every other one
    (section "Unsigned Slice Encoding", first paragraph).  Smallest S with 8+7(S-1) >= bits+1."""
    S = 1
    while 8 + 7 * (S - 1) < bits + 1:
        S += 1
    return S


def slices_dynamic(target_bits: int, esc: int) -> int:
    """ceil((target_bits + ESC + sign + H) / 8)."""
    return max(1, -(-(target_bits + esc + 1 + H) // 8))


def kept_pairs(S: int):
    """(s, t) with s + t <= S - 1, grouped by anti-diagonal d = s + t."""
    return [[(s, d - s) for s in range(d + 1)] for d in range(S)]


@dataclass
class HeuristicModel:
    """Integer cost model for "emulation slower than FP64?" (parity unpinned: own constants).
    Rates in operations per nanosecond, fixed cost in nanoseconds, bandwidth in bytes/ns."""
    int8_ops_per_ns: int = 2650000
    fp64_flops_per_ns: int = 74000
    bytes_per_ns: int = 4000
    fixed_ns: int = 60000

    def emulation_slower(self, S: int, m: int, n: int, k: int, pairs: int | None = None) -> bool:
        """S: slice count (sets the streaming cost); pairs: slice-pair products per tile of C,
        S(S+1)/2 unless the tiles of C take different slice counts (then the mean, rounded up).
        Streamed bytes: the scan reads 8 and the slicing reads 8 and writes S per operand element; per
        element of C the aggregated anti-diagonal sums (4 + (S-1) bytes) are written once and read
        once, and C is read and written."""
        flops = 2 * m * n * k
        if pairs is None:
            pairs = S * (S + 1) // 2
        stream = (16 + S) * (m * k + k * n) + (2 * S + 22) * m * n
        t_emu = self.fixed_ns + (flops // self.int8_ops_per_ns) * pairs + stream // self.bytes_per_ns
        t_f64 = flops // self.fp64_flops_per_ns
        return t_emu > t_f64


@dataclass
class Verdict:
    fallback: int
    reason: int
    slices_used: int        # S; with per-tile slice counts the largest of them
    esc: int
    required_bits: int
    infnan: int
    slices_min: int = 0     # smallest slice count of any tile of C (== slices_used without per-tile counts)
    pair_tiles: int = 0     # slice-pair products of TILE x TILE blocks of C the call multiplies, summed over tiles


def pairs_of(S: int) -> int:
    return S * (S + 1) // 2


def tile_count(m: int, n: int, tile: int = TILE) -> int:
    return (-(-m // tile)) * (-(-n // tile))


def verdict(mode: int, target_bits: int, max_bits: int, slices_override: int, infnan: bool,
            esc: int, m: int, n: int, k: int, heuristic: HeuristicModel | None = None,
            tile_esc: np.ndarray | None = None) -> Verdict:
    """The decision record.  `esc` is -1 when no ESC was computed (unguarded / native modes).
    tile_esc (DYNAMIC only): the ESC of every TILE x TILE block of C (esc_coarse_tiles); each block
    then takes slices_dynamic(target_bits, its own ESC) slices, `esc` must be their maximum, and
    the cost model is fed the mean number of slice-pair products per block.

    DYNAMIC         S from target_bits + ESC; falls back on Inf/NaN, on required_bits >
                    max_bits, or when the heuristic predicts emulation to be slower.
    FORCED_GUARDED  scan and ESC run but S is forced; only Inf/NaN falls back.
    FIXED_GUARDED   S fixed; falls back on Inf/NaN, when target_bits + ESC > max_bits, or when
                    the fixed S slices cannot hold target_bits + ESC (the dynamic rule would
                    ask for more slices than S: with the headroom bit S slices carry 8S - 2
                    magnitude bits, so "55 bits" = 7 slices carry 54).
    FIXED_UNGUARDED S fixed; never falls back.
    NATIVE          always the FP64 GEMM."""
    S_fixed = slices_override if slices_override > 0 else slices_for_bits(max_bits)
    S_fixed = min(S_fixed, MAX_SLICES)
    if mode == MODE_NATIVE:
        return Verdict(1, REASON_NATIVE, 0, -1, 0, 0)
    nt = tile_count(m, n)
    if mode == MODE_FIXED_UNGUARDED:
        return Verdict(0, REASON_NONE, S_fixed, -1, 0, 0, S_fixed, nt * pairs_of(S_fixed))
    if infnan:
        return Verdict(1, REASON_INFNAN, 0, -1, 0, 1)
    required = target_bits + esc
    if mode == MODE_FORCED_GUARDED:
        return Verdict(0, REASON_NONE, S_fixed, esc, required, 0, S_fixed, nt * pairs_of(S_fixed))
    if mode == MODE_FIXED_GUARDED:
        if required > max_bits or slices_dynamic(target_bits, esc) > S_fixed:
            return Verdict(1, REASON_BITS, 0, esc, required, 0)
        return Verdict(0, REASON_NONE, S_fixed, esc, required, 0, S_fixed, nt * pairs_of(S_fixed))
    if mode == MODE_DYNAMIC:
        if required > max_bits:
            return Verdict(1, REASON_BITS, 0, esc, required, 0)
        S = min(slices_dynamic(target_bits, esc), MAX_SLICES)
        if tile_esc is None:
            S_min, pair_tiles = S, nt * pairs_of(S)
        else:
            assert tile_esc.size == nt and int(tile_esc.max()) == esc
            S_t = [min(slices_dynamic(target_bits, int(e)), MAX_SLICES) for e in tile_esc.ravel()]
            S_min, pair_tiles = min(S_t), sum(pairs_of(x) for x in S_t)
        pairs_mean = -(-pair_tiles // nt)                     # rounded up
        if heuristic is not None and heuristic.emulation_slower(S, m, n, k, pairs_mean):
            return Verdict(1, REASON_HEURISTIC, 0, esc, required, 0)
        return Verdict(0, REASON_NONE, S, esc, required, 0, S_min, pair_tiles)
    raise ValueError("unknown mode")


def tile_slices(target_bits: int, tile_esc: np.ndarray) -> np.ndarray:
    """Slice count of every TILE x TILE block of C from its own ESC."""
    f = np.vectorize(lambda e: min(slices_dynamic(target_bits, int(e)), MAX_SLICES))
    return f(tile_esc).astype(np.int64)


def shape_only_fallback(mode: int, target_bits: int, m: int, n: int, k: int,
                        heuristic: HeuristicModel | None) -> bool:
    """DYNAMIC mode with the heuristic on: the ESC is at least 1, so no input can get fewer than
    slices_dynamic(target_bits, 1) slices; if the cost model already calls that count slower than
    the native GEMM, the call goes native without scanning the operands (the record then holds
    no ESC and no Inf/NaN flag).  Own choice within the section "Heuristic run time Selection"
    (small problems fall back to native FP64 so that run time never drops below the baseline)."""
    if mode != MODE_DYNAMIC or heuristic is None:
        return False
    return heuristic.emulation_slower(min(slices_dynamic(target_bits, 1), MAX_SLICES), m, n, k)


# --------------------------------------------------------------------------------------
# O5  exponent-aligned slicing with the unsigned-slice encoding
#     (sections "ESC" on shifting within a row, and "Unsigned Slice Encoding")
# --------------------------------------------------------------------------------------
def remap_unsigned_to_signed(X: int, S: int):
    """Digits d_0..d_{S-1} (d_0 leading), each in [-128,127], with X = sum d_s 256^(S-1-s).

    Follows the paper's description literally: take the S bytes of the two's-complement
    integer X (leading byte signed, the others u8); walking from the least significant byte
    upwards, a u8 byte in [0,127] is kept, a byte in [128,255] becomes byte-256 and the next
    higher byte is incremented."""
    assert -(1 << (8 * S - 1)) <= X < (1 << (8 * S - 1))
    digits = [0] * S
    carry = 0
    for pos in range(S - 1, 0, -1):                 # sub-leading bytes, least significant first
        u = ((X >> (8 * (S - 1 - pos))) & 0xFF) + carry
        if u >= 128:
            digits[pos] = u - 256
            carry = 1
        else:
            digits[pos] = u
            carry = 0
    lead = (X >> (8 * (S - 1))) + carry             # arithmetic shift keeps the sign
    assert -128 <= lead <= 127, "leading digit left the s8 range"
    digits[0] = lead
    return digits


def fixed_point(a: float, e_row: int, S: int) -> int:
    """X = floor(a * 2^q) with q = 8S - 2 - H - e_row, exact (rounding toward -infinity)."""
    if a == 0.0 or e_row <= NEG_INF_BELOW:
        return 0
    q = 8 * S - 2 - H - e_row
    return math.floor(Fraction(a) * (Fraction(2) ** q))


def slice_vector_exact(v: np.ndarray, e_row: int, S: int) -> np.ndarray:
    """S x len(v) int8 digits of one row of A (or one column of B); Python integers, any S."""
    out = np.zeros((S, len(v)), dtype=np.int8)
    for l, a in enumerate(v):
        out[:, l] = remap_unsigned_to_signed(fixed_point(float(a), e_row, S), S)
    return out


def slice_rows_exact(A: np.ndarray, eA: np.ndarray, S: int) -> np.ndarray:
    """S x m x k int8: slices of A aligned per row.  For B pass B.T and eB (gives S x n x k)."""
    m, k = A.shape
    out = np.zeros((S, m, k), dtype=np.int8)
    for i in range(m):
        out[:, i, :] = slice_vector_exact(A[i], int(eA[i]), S)
    return out


def slice_rows_int64(A: np.ndarray, eA: np.ndarray, S: int) -> np.ndarray:
    """Same result as slice_rows_exact for S <= 8, vectorised with 64-bit integers.

    a = sgn * M * 2^(E-1075) with the 53-bit integer significand M, so
    X = floor(sgn * M * 2^(E - 1075 + q)): a left shift when the exponent is non-negative and
    an arithmetic right shift (which rounds toward -infinity) otherwise.  The byte walk of
    remap_unsigned_to_signed is then applied to all entries at once."""
    assert 1 <= S <= 8
    A = np.asarray(A, dtype=np.float64)
    m, k = A.shape
    bits = A.view(np.int64)
    field = (bits >> 52) & 0x7FF
    frac = bits & ((1 << 52) - 1)
    M = np.where(field > 0, frac | (1 << 52), frac)
    M = np.where(bits < 0, -M, M)
    E = np.maximum(field, 1)
    e_row = np.where(eA > NEG_INF_BELOW, eA, 0).astype(np.int64)[:, None]
    sh = E - 1075 + (8 * S - 2 - H) - e_row
    X = np.where(sh >= 0, M << np.clip(sh, 0, 62), M >> np.clip(-sh, 0, 63))
    out = np.zeros((S, m, k), dtype=np.int8)
    carry = np.zeros((m, k), dtype=np.int64)
    for pos in range(S - 1, 0, -1):
        u = ((X >> (8 * (S - 1 - pos))) & 0xFF) + carry
        hi = u >= 128
        out[pos] = np.where(hi, u - 256, u).astype(np.int8)
        carry = hi.astype(np.int64)
    lead = (X >> (8 * (S - 1))) + carry
    assert lead.min(initial=0) >= -128 and lead.max(initial=0) <= 127
    out[0] = lead.astype(np.int8)
    return out


def fixed_point_shift(a: float, e_row: int, S: int) -> int:
    """The same X as fixed_point, by integer shifts instead of rational arithmetic (faster):
    a = mant * 2^(p-53) with the integer mant = frexp-significand * 2^53, so X is mant shifted
    by p - 53 + q; Python's >> on a negative integer rounds toward -infinity."""
    if a == 0.0 or e_row <= NEG_INF_BELOW:
        return 0
    f, p = math.frexp(a)
    mant = int(f * 9007199254740992.0)          # exact: f has at most 53 significant bits
    sh = p - 53 + (8 * S - 2 - H - e_row)
    return mant << sh if sh >= 0 else mant >> (-sh)


def slice_rows_bigint(A: np.ndarray, eA: np.ndarray, S: int) -> np.ndarray:
    """slice_rows_exact with fixed_point_shift; any S, moderate sizes."""
    m, k = A.shape
    out = np.zeros((S, m, k), dtype=np.int8)
    for i in range(m):
        er = int(eA[i])
        for l in range(k):
            out[:, i, l] = remap_unsigned_to_signed(fixed_point_shift(float(A[i, l]), er, S), S)
    return out


def slice_rows(A: np.ndarray, eA: np.ndarray, S: int) -> np.ndarray:
    return slice_rows_int64(A, eA, S) if S <= 8 else slice_rows_bigint(A, eA, S)


# --------------------------------------------------------------------------------------
# O6  slice-pair products with exact integer accumulation  (section "FP64 Emulation on
#     Low-Precision Units"; accumulator overflow: section "Pre-processing and Safety Checks")
# --------------------------------------------------------------------------------------
def k_block_length(S: int) -> int:
    """Longest k-range one int32 accumulator can take: |digit product| <= 2^14 and an
    anti-diagonal sums at most S*k_blk of them; the carry that the aggregation of the less
    significant anti-diagonals brings in (normalised_digits) is below 2^23 in magnitude, so
    S*k_blk*2^14 + 2^23 <= 2^31 - 1, i.e. S*k_blk <= 2^17 - 2^9 - 1; rounded down to a multiple
    of 256."""
    return ((1 << 17) - (1 << 9) - 1) // S // 256 * 256


def slice_products(As: np.ndarray, Bs: np.ndarray) -> np.ndarray:
    """P[kb, d, i, j] = sum_{s+t=d} sum_{l in block kb} As[s,i,l] * Bs[t,j,l]   (int32).

    As is S x m x k, Bs is S x n x k.  The inner matrix product runs in float64, which is
    exact here (every partial sum is an integer below 2^31); the result is asserted to fit
    int32."""
    S, m, k = As.shape
    n = Bs.shape[1]
    kb_len = k_block_length(S)
    nkb = max(1, -(-k // kb_len))
    P = np.zeros((nkb, S, m, n), dtype=np.int64)
    for kb in range(nkb):
        lo, hi = kb * kb_len, min(k, (kb + 1) * kb_len)
        for d, pairs in enumerate(kept_pairs(S)):
            for s, t in pairs:
                prod = As[s, :, lo:hi].astype(np.float64) @ Bs[t, :, lo:hi].astype(np.float64).T
                P[kb, d] += prod.astype(np.int64)
            assert np.abs(P[kb, d]).max(initial=0) < (1 << 31), "int32 accumulator would overflow"
    return P.astype(np.int32)


def slice_products_loops(As: np.ndarray, Bs: np.ndarray) -> np.ndarray:
    """The same as slice_products by a literal loop nest in Python integers (tiny inputs)."""
    S, m, k = As.shape
    n = Bs.shape[1]
    kb_len = k_block_length(S)
    nkb = max(1, -(-k // kb_len))
    P = np.zeros((nkb, S, m, n), dtype=np.int64)
    for kb in range(nkb):
        for d in range(S):
            for s in range(d + 1):
                t = d - s
                for i in range(m):
                    for j in range(n):
                        acc = 0
                        for l in range(kb * kb_len, min(k, (kb + 1) * kb_len)):
                            acc += int(As[s, i, l]) * int(Bs[t, j, l])
                        P[kb, d, i, j] += acc
    assert np.abs(P).max(initial=0) < (1 << 31)
    return P.astype(np.int32)


# --------------------------------------------------------------------------------------
# O7  recomposition to FP64 and alpha/beta  (sections "FP64 Emulation on Low-Precision
#     Units" and "Pre-processing and Safety Checks", second half)
# --------------------------------------------------------------------------------------
def normalised_digits(P: np.ndarray):
    """Aggregates the S anti-diagonal sums of each k-block into one exact integer
    Z = sum_d P_d * 256^(S-1-d), written in base 256 with balanced digits and a leading word:
    Z = T0 * 256^(S-1) + sum_{d>=1} lo_d * 256^(S-1-d),  lo_d in [-128, 127].

    Carries run from the least significant anti-diagonal upwards: T = P_d + carry,
    lo_d = the residue of T modulo 256 that lies in [-128, 127], carry = (T - lo_d) / 256.
    Balanced digits keep a small Z small in every digit (no borrow ripples to the top), so the
    floating-point conversion that follows loses nothing to cancellation.  Every T (and T0) is
    asserted to fit int32: the k-block rule leaves room for the carry.  Returns
    (T0: nkb x m x n int32, lo: nkb x (S-1) x m x n int8, lo[:, d-1] holding lo_d)."""
    nkb, S, m, n = P.shape
    lo = np.zeros((nkb, max(S - 1, 0), m, n), dtype=np.int8)
    carry = np.zeros((nkb, m, n), dtype=np.int64)
    for d in range(S - 1, 0, -1):
        T = P[:, d].astype(np.int64) + carry
        assert np.abs(T).max(initial=0) < (1 << 31) - 128, "int32 accumulator would overflow"
        digit = ((T + 128) & 255) - 128
        lo[:, d - 1] = digit.astype(np.int8)
        carry = (T - digit) >> 8                         # exact division
    T0 = P[:, 0].astype(np.int64) + carry
    assert np.abs(T0).max(initial=0) < (1 << 31), "int32 accumulator would overflow"
    return T0.astype(np.int32), lo


def recompose(P: np.ndarray, eA: np.ndarray, eB: np.ndarray) -> np.ndarray:
    """AB_ij = 2^(eA_i + eB_j + 2H - 12) * sum_kb sum_d 256^-d P[kb,d,i,j].

    The partial results of a k-block are aggregated exactly, in integer form
    (normalised_digits), and converted to FP64 only then, least significant digit first:
    R <- lo_d + R * 2^-8 for d = S-1 .. 1, then R <- T0 + R * 2^-8.  Up to seven slices the
    digits below T0 have at most 48 bits, so every step but the last is exact and the k-block's
    value is the exact integer rounded once; beyond seven, balanced digits keep every partial
    sum within half a unit of its leading digit, so the roundings stay relative to the value
    itself.  k-blocks are added in ascending order in the
    unscaled range; the power-of-two scale is applied last, so an Inf can only appear in this
    terminal conversion."""
    nkb, S, m, n = P.shape
    T0, lo = normalised_digits(P)
    R = np.zeros((m, n), dtype=np.float64)
    for kb in range(nkb):
        Rb = np.zeros((m, n), dtype=np.float64)
        for d in range(S - 1, 0, -1):
            Rb = lo[kb, d - 1].astype(np.float64) + Rb * 2.0 ** -8
        Rb = T0[kb].astype(np.float64) + Rb * 2.0 ** -8
        R = R + Rb
    ea = np.where(eA > NEG_INF_BELOW, eA, 0).astype(np.int64)
    eb = np.where(eB > NEG_INF_BELOW, eB, 0).astype(np.int64)
    scale = ea[:, None] + eb[None, :] + (2 * H - 12)
    with np.errstate(over="ignore", under="ignore"):
        return np.ldexp(R, scale.astype(np.int32))


def recompose_tiles(P: np.ndarray, eA: np.ndarray, eB: np.ndarray, S_tile: np.ndarray,
                    tile: int = TILE) -> np.ndarray:
    """recompose() with a slice count per tile x tile block of C: block (ti, tj) uses the anti-
    diagonals d < S_tile[ti, tj] of P only, i.e. the leading S_tile digits of every row of A and
    column of B and the pairs s + t <= S_tile - 1.  The digits are those of the one decomposition
    into max(S_tile) slices: its leading S' digits represent the entry to within 0.51 units of
    digit S' (the dropped tail is a signed number), which is what S' slices need to deliver."""
    nkb, S, m, n = P.shape
    out = np.zeros((m, n), dtype=np.float64)
    for ti in range(S_tile.shape[0]):
        for tj in range(S_tile.shape[1]):
            r = slice(ti * tile, min(m, (ti + 1) * tile))
            c = slice(tj * tile, min(n, (tj + 1) * tile))
            out[r, c] = recompose(P[:, :int(S_tile[ti, tj]), r, c], eA[r], eB[c])
    return out


def axpby(alpha: float, AB: np.ndarray, beta: float, C: np.ndarray | None) -> np.ndarray:
    """alpha*AB + beta*C with every product and the sum rounded separately; C is not read
    when beta == 0."""
    with np.errstate(over="ignore", invalid="ignore"):
        out = np.float64(alpha) * AB
        if beta != 0.0:
            out = out + np.float64(beta) * np.asarray(C, dtype=np.float64)
    return out


# --------------------------------------------------------------------------------------
# the whole call
# --------------------------------------------------------------------------------------
@dataclass
class Trace:
    verdict: Verdict
    eA: np.ndarray | None = None
    eB: np.ndarray | None = None
    As: np.ndarray | None = None       # S x m x k
    Bs: np.ndarray | None = None       # S x n x k
    P: np.ndarray | None = None        # nkb x S x m x n
    C: np.ndarray | None = None
    S_tile: np.ndarray | None = None   # slice count per TILE x TILE block of C (per-tile mode only)


def native_gemm(alpha, A, B, beta, C):
    """The FP64 fallback: an ordinary matrix product (low bits depend on summation order)."""
    with np.errstate(all="ignore"):
        AB = np.asarray(A, dtype=np.float64) @ np.asarray(B, dtype=np.float64)
    return axpby(alpha, AB, beta, C)


def emulated_dgemm(A: np.ndarray, B: np.ndarray, alpha: float = 1.0, beta: float = 0.0,
                   C: np.ndarray | None = None, *, mode: int = MODE_FORCED_GUARDED,
                   target_bits: int = 53, max_bits: int = 55, slices: int = 0,
                   esc_block: int = DEFAULT_ESC_BLOCK,
                   heuristic: HeuristicModel | None = None, keep: bool = True,
                   per_tile: bool = False, tile: int = TILE) -> Trace:
    """C = alpha*A*B + beta*C through the decision process of the paper's flowchart:
    CheckInfNaN(A), CheckInfNaN(B) -> ESC(A,B) -> verdict -> emulated or native GEMM.
    per_tile (DYNAMIC only): every tile x tile block of C takes the slice count of its own ESC
    (`tile` other than TILE is for small test cases; the verdict's tile counts assume TILE)."""
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    m, k = A.shape
    n = B.shape[1]
    if m == 0 or n == 0 or k == 0 or alpha == 0.0:     # BLAS convention: C <- beta*C
        out = np.zeros((m, n)) if beta == 0.0 else np.float64(beta) * np.asarray(C, dtype=np.float64)
        return Trace(Verdict(0, REASON_NONE, 0, -1, 0, 0), C=out)
    if shape_only_fallback(mode, target_bits, m, n, k, heuristic):
        return Trace(Verdict(1, REASON_HEURISTIC, 0, -1, 0, 0), C=native_gemm(alpha, A, B, beta, C))
    guarded = mode in (MODE_DYNAMIC, MODE_FORCED_GUARDED, MODE_FIXED_GUARDED)
    infnan = guarded and (has_inf_nan(A) or has_inf_nan(B))
    tiled = per_tile and mode == MODE_DYNAMIC and guarded and not infnan
    tile_esc = esc_coarse_tiles(A, B, esc_block, tile) if tiled else None
    if tiled:
        esc = int(tile_esc.max())
    else:
        esc = esc_coarse(A, B, esc_block) if (guarded and not infnan) else -1
    v = verdict(mode, target_bits, max_bits, slices, infnan, esc, m, n, k, heuristic,
                tile_esc if (tiled and tile == TILE) else None)
    if v.fallback:
        return Trace(v, C=native_gemm(alpha, A, B, beta, C))
    S = v.slices_used
    eA, eB = row_exponents(A), col_exponents(B)
    As = slice_rows(A, eA, S)
    Bs = slice_rows(np.ascontiguousarray(B.T), eB, S)
    P = slice_products(As, Bs)
    S_tile = tile_slices(target_bits, tile_esc) if tiled else None
    AB = recompose_tiles(P, eA, eB, S_tile, tile) if tiled else recompose(P, eA, eB)
    out = axpby(alpha, AB, beta, C)
    if keep:
        return Trace(v, eA, eB, As, Bs, P, out, S_tile)
    return Trace(v, C=out, S_tile=S_tile)


# --------------------------------------------------------------------------------------
# complex product by the 4M method  (section "Conclusion": the emulation, guardrails included,
# extends to ZGEMM via 4M: four real matrix products on the real and imaginary parts)
# --------------------------------------------------------------------------------------
def emulated_zgemm(A: np.ndarray, B: np.ndarray, alpha: complex = 1.0, beta: complex = 0.0,
                   C: np.ndarray | None = None, **kw):
    """C = alpha*A*B + beta*C for complex matrices: with A = Ar + i Ai, B = Br + i Bi,

        Pr = Ar Br - Ai Bi,        Pi = Ar Bi + Ai Br,

    each of the four real products one emulated_dgemm call (its own scan, ESC and verdict; keyword
    arguments are passed through), the second product of each pair accumulating onto the first
    (alpha = -1 or +1, beta = 1).  Then  C = alpha*(Pr + i Pi) + beta*C  with every real product and
    sum rounded separately, in the order written below; C is not read when beta == 0.
    Returns (C, [the four verdicts in the order Ar Br, Ai Bi, Ar Bi, Ai Br])."""
    A = np.asarray(A, dtype=np.complex128)
    B = np.asarray(B, dtype=np.complex128)
    Ar, Ai = np.ascontiguousarray(A.real), np.ascontiguousarray(A.imag)
    Br, Bi = np.ascontiguousarray(B.real), np.ascontiguousarray(B.imag)
    kw = dict(kw, keep=False)
    t1 = emulated_dgemm(Ar, Br, 1.0, 0.0, None, **kw)
    t2 = emulated_dgemm(Ai, Bi, -1.0, 1.0, t1.C, **kw)
    t3 = emulated_dgemm(Ar, Bi, 1.0, 0.0, None, **kw)
    t4 = emulated_dgemm(Ai, Br, 1.0, 1.0, t3.C, **kw)
    Pr, Pi = t2.C, t4.C
    ar, ai = np.float64(complex(alpha).real), np.float64(complex(alpha).imag)
    br, bi = np.float64(complex(beta).real), np.float64(complex(beta).imag)
    with np.errstate(over="ignore", invalid="ignore"):
        out_r = ar * Pr - ai * Pi
        out_i = ar * Pi + ai * Pr
        if beta != 0.0:
            Cr, Ci = np.asarray(C).real, np.asarray(C).imag
            out_r = out_r + (br * Cr - bi * Ci)
            out_i = out_i + (br * Ci + bi * Cr)
    return out_r + 1j * out_i, [t1.verdict, t2.verdict, t3.verdict, t4.verdict]
