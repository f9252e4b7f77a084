// Slice-pair INT8 GEMMs with exact int32 accumulation: the one dense contraction of the method.
// (paper: section "FP64 Emulation on Low-Precision Units": products are computed slice by slice;
//  section "ESC": cost is quadratic in the slice count; the kept pairs are s + t <= S - 1, the
//  count behind "seven slices rather than eight: 22 % less compute"; section "Pre-processing
//  and Safety Checks": partial results are aggregated so that accumulators cannot overflow.)
//
//   P_d[j][i] = sum_{s+t=d} sum_{l in k-block kb} As[s][i][l] * Bs[t][j][l],   d = 0..S-1
//
// One launch covers all S(S+1)/2 pairs: a workgroup owns a 256x256 tile of C and walks the
// anti-diagonals d from the least significant (S-1) to the most significant (0); all pairs of one d
// accumulate into the same int32 registers (their k ranges are simply concatenated).  When an
// anti-diagonal is complete its sum T is split exactly into a balanced digit (T mod 256 in
// [-128,127], one byte per element, written out) and a carry (T - digit)/256 that stays in the
// accumulators as the start value of the next anti-diagonal; the last one (d = 0) is written as an
// int32 word.  So a k-block leaves the exact integer sum_d P_d 256^(S-1-d) in 4 + (S-1) bytes per
// element instead of 4S, already aggregated: the FP64 recomposition converts it in one pass.
//
// Mapping to gfx950:
//  * v_mfma_i32_32x32x32_i8; 4 waves per workgroup, each wave a 128x128 sub-tile (4x4 MFMA
//    tiles, 256 accumulator registers per lane); one workgroup per CU.
//  * K step 64 per pipeline stage; 4 LDS stages of 32 KB (128 of the CU's 160 KB).  Tiles go
//    from HBM/L2 straight into LDS with global_load_lds_dwordx4 (no staging registers, no LDS
//    store instructions), issued three stages ahead of their use; one workgroup barrier per
//    stage.  The slice panels are stored [k/16][row][16], so a tile is four contiguous 4 KB
//    runs per operand and the LDS image [k chunk][row][16 B] is what the MFMA operand loads
//    read (ds_read_b128 per lane: row = lane%32, k chunk = lane/32) without bank conflicts.
//  * The B-slices feed the MFMA's row operand and the A-slices its column operand, so the lane
//    index of the result runs along i and the stores to P (i contiguous) coalesce.
//  * Workgroup ids are remapped so that the tiles resident on one XCD form a compact block and
//    share their A and B panels in that XCD's L2; the workgroups of such a block wait for each
//    other (bounded) so that they stay within what L2 holds.
//  * One wave per SIMD, so nothing hides an instruction that delays the next MFMA: at most one
//    LDS read or one tile transfer (three instructions) sits between two MFMAs, tile addresses
//    advance by one add per K step (the full address is recomputed only when the slice pair
//    changes), and the workgroup barrier of a K step is followed by four MFMAs that cover it.
#include "oz_internal.h"

namespace oz {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBM = 256;             // tile extent along i (rows of op(A))
constexpr int kBN = 256;             // tile extent along j (columns of op(B))
constexpr int kBK = 64;              // K step per pipeline stage (kKPad is a multiple)
constexpr int kStages = 4;
constexpr int kStageBytes = (kBM + kBN) * kBK;   // 32 KB
constexpr int kGemmLds = kStages * kStageBytes;  // 128 KB
constexpr int kDmaPerStage = 2 * (kBK / 16);     // DMA instructions per wave per stage (A and B)
static_assert(kKPad % kBK == 0, "k padding must cover whole K steps");
static_assert(kBM == kTile && kBN == kTile, "a workgroup tile is one block of C with its own slice count");
static_assert(kDmaPerStage == 8, "the vmcnt immediates below assume 8 DMA instructions per stage");

constexpr int kRoundTiles = 32;       // workgroups an XCD runs at a time: 32 CUs, one workgroup each
constexpr int kMaxSyncSpins = 384;    // upper bound of the wait for the other workgroups of a round
constexpr int kMidSyncMinK = 12288;   // from this k on, workgroups also wait after every anti-diagonal
constexpr int kMinSplitSteps = 8;     // a part of a split k range keeps at least this many K steps

// Records this workgroup's arrival at *counter and, if `wait`, waits (bounded, about half a
// millisecond) until `target` workgroups have arrived.  The wait only improves cache locality:
// correctness does not depend on it, and every wave gets past it whatever the other workgroups do.
// Returns whether the others were met in time; a workgroup that was not (the chip is shared with
// another kernel, or workgroups are not placed as assumed) keeps counting its arrivals, which the
// others rely on, but stops waiting, so the cost of a wrong assumption is paid once per tile.
__device__ __forceinline__ bool round_sync(int32_t* counter, int target, bool wait) {
    int met = 0;
    if (threadIdx.x == 0) {
        atomicAdd(counter, 1);
        if (wait) {
            for (int spin = 0; spin < kMaxSyncSpins && !met; ++spin) {
                met = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target;
                if (!met) __builtin_amdgcn_s_sleep(8);
            }
        }
    }
    return __syncthreads_or(met) != 0;
}

__device__ __forceinline__ v4i as_v4i(const uint4& v) { return v4i{int(v.x), int(v.y), int(v.z), int(v.w)}; }

// linear workgroup id -> tile coordinates.  Ids are dealt round-robin to the 8 XCDs by the
// hardware; each XCD is given a contiguous range of a tile order in which 32 consecutive tiles
// form a 4 (i) x 8 (j) block.
// position `lin` of the tile order -> tile coordinates: panels of 8 tile columns, i fastest inside
__device__ __forceinline__ void lin_to_tile(int lin, int nti, int ntj, int& ti, int& tj) {
    constexpr int GW = 8;
    const int panel = lin / (GW * nti);
    const int in_panel = lin - panel * GW * nti;
    const int w = min(GW, ntj - panel * GW);
    ti = in_panel / w;
    tj = panel * GW + in_panel % w;
}

// A launch covers the tiles [tile_begin, tile_begin + tile_count) of the tile order.  With a k split
// (zsplit > 1) a work unit is (tile, part of the k range); units are ordered part by part, so the
// units an XCD runs together still are neighbouring tiles of the same k range.
// `order` (per-tile mode, else null) maps a position of the tile order to the tile that runs there.
__device__ __forceinline__ void tile_of(int bid, int nti, int ntj, int tile_begin, int tile_count, int zsplit,
                                        const int32_t* __restrict__ order,
                                        int& ti, int& tj, int& z, int& xcd, int& slot, int& xcd_tiles, int& lin) {
    const int total = tile_count * zsplit;
    xcd = bid & 7;
    slot = bid >> 3;
    const int per = total >> 3, rem = total & 7;
    xcd_tiles = per + (xcd < rem ? 1 : 0);
    const int unit = xcd * per + min(xcd, rem) + slot;
    z = unit / tile_count;
    lin = tile_begin + unit - z * tile_count;
    lin_to_tile(order ? order[lin] : lin, nti, ntj, ti, tj);
}

// 64 lanes x 16 B from global memory into LDS: lane l's 16 bytes land at lds_addr + LDS_IMM + 16*l.
// The LDS byte address travels in M0 (set by the scalar add).  The compiler does not see this as a
// memory access, so completion is awaited with explicit s_waitcnt vmcnt(...) below.
// The global address is a wave-uniform base (scalar registers) plus a per-lane byte offset
// (lane position plus the k chunk's distance, loop-invariant), so stepping through the tiles
// costs two scalar adds per K step.
template <int LDS_IMM>
__device__ __forceinline__ void dma16(const uint8_t* gbase, uint32_t lane_off, uint32_t lds_addr) {
    asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(lane_off), "s"(gbase), "n"(LDS_IMM) : "memory", "scc");
}

// One dword per lane to a wave-uniform base (scalar register pair) plus a 32-bit per-lane byte offset.
// Written as assembly so that the address stays in this form: left to itself the compiler builds a
// 64-bit per-lane address for each of the several hundred stores of an epilogue, hoists them out of
// the anti-diagonal loop and spills them.
// The s_nop covers the five wait states the hardware needs between a vector-ALU write of a scalar
// register (a register-allocator reload with v_readlane, say) and a memory instruction that reads
// it as its base: inside an asm block the compiler does not insert them itself, and a store issued
// too early takes the stale register value as its address.
__device__ __forceinline__ void store_lane_dword(void* uniform_base, uint32_t lane_byte_off, uint32_t data) {
    asm volatile("s_nop 4\n\tglobal_store_dword %0, %1, %2"
                 :: "v"(lane_byte_off), "v"(data), "s"(uniform_base) : "memory");
}

// SPLIT: the launch splits the k range of its tiles over several workgroups (zsplit > 1)
template <bool SPLIT>
__global__ __launch_bounds__(256) void gemm_i8_kernel(const int8_t* __restrict__ As,
                                                      const int8_t* __restrict__ Bs,
                                                      int32_t* __restrict__ T, int8_t* __restrict__ L,
                                                      int32_t* __restrict__ raw, int raw_slots,
                                                      int64_t mp, int64_t np, int64_t kp, int s_cap,
                                                      Record* rec, int full_chip, int zsplit,
                                                      int tile_begin, int tile_count,
                                                      const int32_t* __restrict__ tile_S) {
    extern __shared__ __align__(16) uint8_t lds[];
    if (rec->res.fallback) return;
    const int S_all = rec->res.slices_used;
    // k-range one int32 accumulator can take with S slices (S*kblk digit products of at most 2^14);
    // the k-blocks are those of the call's largest slice count, whatever this tile's own count is
    const int64_t kblk = k_block_length(S_all);
    const int nkb = int((kp + kblk - 1) / kblk);

    int ti, tj, z, xcd, slot, xcd_tiles, unit_tile;   // unit_tile: this tile's position in the tile order
    // per-tile mode: the table of slice counts is followed by the order the tiles are dealt in
    const int32_t* order = tile_S ? tile_S + int(mp / kBM) * int(np / kBN) : nullptr;
    tile_of(blockIdx.x, int(mp / kBM), int(np / kBN), tile_begin, tile_count, zsplit, order, ti, tj, z, xcd, slot,
            xcd_tiles, unit_tile);
    // slice count of this tile of C: its own (per-tile mode: the first S digit planes of the operands
    // and the pairs s + t <= S - 1) or the call's
    const int S = tile_S ? min(tile_S[tj * int(mp / kBM) + ti], S_all) : S_all;

    // This workgroup's share of the K steps: part z of zsplit equal parts of the whole k range (one
    // part = everything when the call has enough tiles to fill the chip).  Parts of the same k-block
    // add their unaggregated anti-diagonal sums into the tile's slot of the raw buffer with integer
    // atomics: exact and order-free.  The host zeroes the slots before such a launch and aggregates
    // them afterwards (aggregate_raw_kernel) into the same T / L form the unsplit tiles write.
    const int kt_total = int(kp / kBK);
    const int kt_first = int(int64_t(kt_total) * z / zsplit);
    const int kt_end = int(int64_t(kt_total) * (z + 1) / zsplit);
    const int kt_per_block = int(kblk / kBK);
    const int kb_first = kt_first / kt_per_block, kb_last = (kt_end - 1) / kt_per_block;

    // Keep the workgroups that share panels in step.  An XCD runs 32 workgroups at a time (one
    // per CU) and its tiles are ordered so that each such round is one 4x8 block.  The workgroups
    // of a round wait for each other at the start of the tile and, when k is long, after every
    // anti-diagonal, because workgroups that have drifted apart never fall back into step by
    // themselves and then miss in L2 what their neighbours loaded (measured at 16384^3 without
    // this: hit rate 49 % instead of 81 %, 10 % more time; at k = 8192 the start of the tile is
    // enough and the extra waits would cost 1 %).  Arrival number q of a workgroup of round r waits
    // for 32*r*steps + (q+1)*members arrivals on the XCD's counter (earlier rounds are full rounds).
    const int sync_steps = (kp >= kMidSyncMinK && !SPLIT) ? nkb * S_all : 1;
    const int sync_round = slot / kRoundTiles;
    const int sync_members = min(kRoundTiles, xcd_tiles - sync_round * kRoundTiles);
    const int sync_base = sync_round * kRoundTiles * sync_steps;
    const bool sync_on = full_chip && xcd_tiles > kRoundTiles && sync_members > 1;
    int sync_q = 0;
    bool sync_wait = true;
    if (sync_on) sync_wait = round_sync(&rec->tile_sync[xcd], sync_base + (++sync_q) * sync_members, sync_wait);

    const int64_t i0 = int64_t(ti) * kBM, j0 = int64_t(tj) * kBN;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wi = wave & 1, wj = wave >> 1;

    v16i acc[4][4];   // [fj][fi]
    const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = zero;

    // K steps [kt_lo(kb), kt_lo(kb) + kt_count(kb)) of k-block kb belong to this workgroup
    auto kt_lo = [&](int kb) -> int { return max(kb * kt_per_block, kt_first); };
    auto kt_count = [&](int kb) -> int { return min((kb + 1) * kt_per_block, kt_end) - kt_lo(kb); };

    // (nkb_, nd, ns, nkt) walks the (k-block, anti-diagonal, pair, K step) sequence ahead of the
    // compute, so the prefetch runs across pair and anti-diagonal boundaries without a bubble.
    // After the last tile it stays put: the surplus transfers land in stages nobody reads again.
    int nkb_ = kb_first, nd = S - 1, ns = 0, nkt = 0;
    int nxt_ktc = kt_count(kb_first);
    int issue_stage = 0;
    const uint32_t lds_base = uint32_t(uintptr_t((__attribute__((address_space(3))) uint8_t*)lds));
    const uint8_t* gA = reinterpret_cast<const uint8_t*>(As) + (i0 + wave * 64) * 16;   // wave-uniform
    const uint8_t* gB = reinterpret_cast<const uint8_t*>(Bs) + (j0 + wave * 64) * 16;
    const uint32_t lane_off = uint32_t(lane) * 16;
    // per-lane byte offsets of the four k chunks of a tile (chunk q is q*rows*16 bytes further on)
    uint32_t offA[4], offB[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        offA[q] = lane_off + uint32_t(q) * uint32_t(mp) * 16u;
        offB[q] = lane_off + uint32_t(q) * uint32_t(np) * 16u;
    }
    const int64_t planeA = kp * mp, planeB = kp * np;   // bytes per slice plane

    // addresses of the next tile to fetch (8 transfers per wave: 4 k chunks of A, 4 of B).  The
    // pointers advance by one K step per tile; only when the pair changes are they recomputed from
    // the iterator (once per k-block length, outside the common path).
    const uint8_t* pa = gA + int64_t(kt_first) * (kBK / 16) * mp * 16;
    const uint8_t* pb = gB + int64_t(S - 1) * (kp * np) + int64_t(kt_first) * (kBK / 16) * np * 16;   // pair (0, S-1)
    const int64_t stepA = int64_t(kBK) * mp, stepB = int64_t(kBK) * np;   // bytes per K step
    uint32_t la;
#define OZ_TILE_ADDR()                                                                           \
    { la = lds_base + issue_stage * kStageBytes + wave * 1024; }
// transfer number x (0..7) of the tile addressed by pa / pb / la
#define OZ_DMA(x)                                                                                \
    {                                                                                            \
        switch (x) {                                                                             \
            case 0: dma16<0 * (kBM * 16)>(pa, offA[0], la); break;                                   \
            case 1: dma16<kBM * kBK + 0 * (kBN * 16)>(pb, offB[0], la); break;                       \
            case 2: dma16<1 * (kBM * 16)>(pa, offA[1], la); break;                                   \
            case 3: dma16<kBM * kBK + 1 * (kBN * 16)>(pb, offB[1], la); break;                       \
            case 4: dma16<2 * (kBM * 16)>(pa, offA[2], la); break;                                   \
            case 5: dma16<kBM * kBK + 2 * (kBN * 16)>(pb, offB[2], la); break;                       \
            case 6: dma16<3 * (kBM * 16)>(pa, offA[3], la); break;                                   \
            default: dma16<kBM * kBK + 3 * (kBN * 16)>(pb, offB[3], la); break;                      \
        }                                                                                        \
    }
#define OZ_TILE_ADVANCE()                                                                        \
    {                                                                                            \
        issue_stage = (issue_stage + 1) & (kStages - 1);                                         \
        if (++nkt == nxt_ktc) {                                                                  \
            nkt = 0;                                                                             \
            if (++ns > nd) {                                                                     \
                ns = 0;                                                                          \
                if (--nd < 0) {                                                                  \
                    nd = S - 1;                                                                  \
                    if (++nkb_ > kb_last) nkb_ = kb_last;                                        \
                    nxt_ktc = kt_count(nkb_);                                                    \
                }                                                                                \
            }                                                                                    \
            const int64_t kc = int64_t(kt_lo(nkb_)) * (kBK / 16);                                \
            pa = gA + int64_t(ns) * planeA + kc * mp * 16;                                       \
            pb = gB + int64_t(nd - ns) * planeB + kc * np * 16;                                  \
        } else {                                                                                 \
            pa += stepA;                                                                         \
            pb += stepB;                                                                         \
        }                                                                                        \
    }
#define OZ_ISSUE_TILE()                                                                          \
    {                                                                                            \
        OZ_TILE_ADDR();                                                                          \
        _Pragma("unroll") for (int x = 0; x < 8; ++x) OZ_DMA(x);                                 \
        OZ_TILE_ADVANCE();                                                                       \
    }
// operand fragment f of K sub-step kk (0 or 1) of the tile in LDS stage `stage`
#define OZ_READ_A(dst, stage, kk, f)                                                             \
    dst[f] = as_v4i((reinterpret_cast<const uint4*>(lds + (stage) * kStageBytes) + wi * 128 +    \
                     (lane & 31) + ((kk) * 2 + (lane >> 5)) * kBM)[(f) * 32])
#define OZ_READ_B(dst, stage, kk, f)                                                             \
    dst[f] = as_v4i((reinterpret_cast<const uint4*>(lds + (stage) * kStageBytes + kBM * kBK) +   \
                     wj * 128 + (lane & 31) + ((kk) * 2 + (lane >> 5)) * kBN)[(f) * 32])
#define OZ_READ_FRAGS(dstA, dstB, stage, kk)                                                     \
    _Pragma("unroll") for (int f = 0; f < 4; ++f) {                                              \
        OZ_READ_A(dstA, stage, kk, f);                                                           \
        OZ_READ_B(dstB, stage, kk, f);                                                           \
    }
#define OZ_MFMA(srcA, srcB, fj, fi)                                                              \
    acc[fj][fi] = __builtin_amdgcn_mfma_i32_32x32x32_i8(srcB[fj], srcA[fi], acc[fj][fi], 0, 0, 0)

    // prologue: three tiles in flight, then wait for the first, publish it, issue the fourth
    OZ_ISSUE_TILE();
    OZ_ISSUE_TILE();
    OZ_ISSUE_TILE();
    asm volatile("s_waitcnt vmcnt(16)\n\ts_barrier" ::: "memory");
    OZ_TILE_ADDR();
#pragma unroll
    for (int x = 0; x < 8; ++x) OZ_DMA(x);   // the iterator moves on in the first half of the loop body
    v4i fa0[4], fb0[4], fa1[4], fb1[4];
    int stage = 0;
    OZ_READ_FRAGS(fa0, fb0, stage, 0);

    for (int kb = kb_first; kb <= kb_last; ++kb) {
        const int ktc = kt_count(kb);
        for (int d = S - 1; d >= 0; --d) {
            const int n_iter = (d + 1) * ktc;
            for (int it = 0; it < n_iter; ++it) {
                // invariant here: transfers of the next three tiles are in flight (24 per wave);
                // fragments of sub-step 0 of the current tile are in fa0/fb0
                // first half: MFMAs of sub-step 0; the LDS reads of sub-step 1 ride along
                // first half: MFMAs of sub-step 0 (16); one LDS read of sub-step 1 after each of the
                // first eight, so that all have returned well before the barrier
#pragma unroll
                for (int q = 0; q < 12; ++q) {
                    OZ_MFMA(fa0, fb0, q >> 2, q & 3);
                    __builtin_amdgcn_sched_barrier(0);
                    if (q < 8) {
                        if (q & 1) { OZ_READ_B(fb1, stage, 1, q >> 1); } else { OZ_READ_A(fa1, stage, 1, q >> 1); }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (q == 9) {   // a gap without memory work: move the iterator past the tile issued last
                        OZ_TILE_ADVANCE();
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                // next tile landed (own transfers), every LDS read of this tile returned; after the
                // barrier that holds for all waves, so this stage may be overwritten.  The last four
                // MFMAs of the first half cover the barrier.
                asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)\n\ts_barrier" ::: "memory");
                const int next_stage = (stage + 1) & (kStages - 1);
                OZ_TILE_ADDR();
#pragma unroll
                for (int q = 12; q < 16; ++q) {
                    OZ_MFMA(fa0, fb0, q >> 2, q & 3);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // second half: MFMAs of sub-step 1; after each one either an LDS read of the next
                // tile's sub-step 0 or a transfer of the tile three stages ahead
#pragma unroll
                for (int g = 0; g < 8; ++g) {
                    OZ_MFMA(fa1, fb1, g >> 1, (g & 1) * 2);
                    __builtin_amdgcn_sched_barrier(0);
                    if (g & 1) { OZ_READ_B(fb0, next_stage, 0, g >> 1); } else { OZ_READ_A(fa0, next_stage, 0, g >> 1); }
                    __builtin_amdgcn_sched_barrier(0);
                    OZ_MFMA(fa1, fb1, g >> 1, (g & 1) * 2 + 1);
                    __builtin_amdgcn_sched_barrier(0);
                    OZ_DMA(g);
                    __builtin_amdgcn_sched_barrier(0);
                }
                stage = next_stage;
            }

            // anti-diagonal d of k-block kb is complete.
            // result register r of MFMA tile (fj, fi): j = fj*32 + 8*(r/4) + 4*(lane/32) + r%4,
            // i = fi*32 + lane%32.  Every address below is a wave-uniform pointer (scalar arithmetic)
            // plus one per-lane 32-bit element offset that is the same for all stores of a kind.
            // the row stride as a value the compiler cannot trace out of this iteration: otherwise the row
            // addresses of all stores (loop-invariant offsets) are hoisted out of the anti-diagonal loop
            // and kept alive, several hundred registers' worth, across the MFMA loop
            int64_t mp_here = mp;
            asm volatile("" : "+s"(mp_here));
            if (SPLIT) {
                // this workgroup holds a part of the k range: add the partial sums into the tile's raw slot
                int32_t* dst = raw + ((int64_t(kb) * s_cap + d) * raw_slots + (unit_tile - tile_begin)) * (kBM * kBN) +
                               (wj * 128) * kBM + wi * 128;
                const uint32_t lane_raw = uint32_t(4 * (lane >> 5)) * kBM + uint32_t(lane & 31);
#pragma unroll
                for (int fj = 0; fj < 4; ++fj)
#pragma unroll
                    for (int fi = 0; fi < 4; ++fi) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            atomicAdd(dst + ((fj * 32 + 8 * (r >> 2) + (r & 3)) * kBM + fi * 32) + lane_raw, acc[fj][fi][r]);
                        acc[fj][fi] = zero;
                    }
            } else if (d > 0) {
                // balanced digit out (the low byte of T is its two's-complement form), carry stays: four
                // consecutive j of one i make a dword, so the lanes of a half-wave write 128 contiguous bytes
                uint32_t* dst = reinterpret_cast<uint32_t*>(L) +
                                ((int64_t(kb) * (s_cap - 1) + (d - 1)) * (np / 4) + (j0 + wj * 128) / 4) * mp + i0 + wi * 128;
                const uint32_t lane_L = (uint32_t(lane >> 5) * uint32_t(mp) + uint32_t(lane & 31)) * 4u;   // bytes
                const v4i zero4 = {0, 0, 0, 0};
#pragma unroll
                for (int fj = 0; fj < 4; ++fj)
#pragma unroll
                    for (int fi = 0; fi < 4; ++fi) {
                        const v16i t = acc[fj][fi];
                        v16i carry;
#pragma unroll
                        for (int rq = 0; rq < 4; ++rq) {
                            const uint32_t w = (uint32_t(t[4 * rq]) & 255u) | ((uint32_t(t[4 * rq + 1]) & 255u) << 8) |
                                               ((uint32_t(t[4 * rq + 2]) & 255u) << 16) | (uint32_t(t[4 * rq + 3]) << 24);
                            store_lane_dword(dst + (int64_t(fj * 8 + 2 * rq) * mp_here + fi * 32), lane_L, w);
                        }
#pragma unroll
                        for (int r = 0; r < 16; ++r) carry[r] = (t[r] + 128) >> 8;
                        // The carries go back into the accumulator tile as the result of a matrix instruction
                        // with zero operands (0*0 + carry).  Written by the vector ALU instead, the tile
                        // would be kept in the ordinary vector registers by the register allocator, and
                        // sixteen such tiles do not fit there beside the loop's own registers.
                        acc[fj][fi] = __builtin_amdgcn_mfma_i32_32x32x32_i8(zero4, zero4, carry, 0, 0, 0);
                    }
            } else {
                // the leading word; the next k-block starts from zero
                int32_t* dst = T + (int64_t(kb) * np + j0 + wj * 128) * mp + i0 + wi * 128;
                const uint32_t lane_T = (uint32_t(4 * (lane >> 5)) * uint32_t(mp) + uint32_t(lane & 31)) * 4u;   // bytes
#pragma unroll
                for (int fj = 0; fj < 4; ++fj)
#pragma unroll
                    for (int fi = 0; fi < 4; ++fi) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            store_lane_dword(dst + (int64_t(fj * 32 + 8 * (r >> 2) + (r & 3)) * mp_here + fi * 32), lane_T,
                                             uint32_t(acc[fj][fi][r]));
                        }
                        acc[fj][fi] = zero;
                    }
            }
            if (sync_on && sync_q < sync_steps)
                sync_wait = round_sync(&rec->tile_sync[xcd], sync_base + (++sync_q) * sync_members, sync_wait);
            // The operand fragments of the next K step were read during the last one, as in every K
            // step; reading them again here (eight LDS reads per anti-diagonal) ends their lifetime
            // before the epilogue above, which needs the registers to pass the accumulators through.
            OZ_READ_FRAGS(fa0, fb0, stage, 0);
        }
    }
    // a tile with fewer anti-diagonals than the call's largest count still owes the round its
    // remaining arrivals: the workgroups that walk more of them count on every member
    if (sync_on && sync_q < sync_steps && threadIdx.x == 0) atomicAdd(&rec->tile_sync[xcd], sync_steps - sync_q);
    // drain the surplus transfers before the workgroup's LDS is released
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

#undef OZ_ISSUE_TILE
#undef OZ_READ_FRAGS
#undef OZ_MFMA
#undef OZ_DMA
#undef OZ_TILE_ADDR
#undef OZ_TILE_ADVANCE
#undef OZ_READ_A
#undef OZ_READ_B

// raw = 0 on the slots of a launch whose workgroups add their parts of the k range into them.
// grid (tiles of the launch, planes); a workgroup clears one 256 x 256 slot of one plane.
__global__ __launch_bounds__(256) void zero_raw_kernel(int32_t* __restrict__ raw, int raw_slots, const Record* rec) {
    if (rec->res.fallback) return;
    int4* base = reinterpret_cast<int4*>(raw + (int64_t(blockIdx.y) * raw_slots + blockIdx.x) * (kBM * kBN));
    for (int v = threadIdx.x; v < kBM * kBN / 4; v += 256) base[v] = make_int4(0, 0, 0, 0);
}

// Aggregates the raw anti-diagonal sums of the split tiles of a launch into the T / L form the unsplit
// tiles write directly: the same integer carry chain, least significant anti-diagonal first.
// grid (tiles of the launch, k-blocks); thread = one i of the tile, walking j four at a time.
__global__ __launch_bounds__(256) void aggregate_raw_kernel(const int32_t* __restrict__ raw, int raw_slots,
                                                            int32_t* __restrict__ T, int8_t* __restrict__ L,
                                                            int64_t mp, int64_t np, int64_t kp, int s_cap, int nti,
                                                            int ntj, int tile_begin, const Record* rec,
                                                            const int32_t* __restrict__ tile_S) {
    if (rec->res.fallback) return;
    const int S_all = rec->res.slices_used;
    const int nkb = int((kp + k_block_length(S_all) - 1) / k_block_length(S_all));
    const int kb = blockIdx.y;
    if (kb >= nkb) return;
    int ti, tj;
    const int pos = tile_begin + int(blockIdx.x);
    lin_to_tile(tile_S ? tile_S[nti * ntj + pos] : pos, nti, ntj, ti, tj);
    const int S = tile_S ? min(tile_S[tj * nti + ti], S_all) : S_all;
    const int il = threadIdx.x;
    const int64_t i = int64_t(ti) * kBM + il, j0 = int64_t(tj) * kBN;
    const int32_t* src = raw + (int64_t(kb) * s_cap * raw_slots + blockIdx.x) * (kBM * kBN) + il;
    const int64_t plane = int64_t(raw_slots) * (kBM * kBN);
    for (int jl4 = 0; jl4 < kBN / 4; ++jl4) {
        int carry[4] = {0, 0, 0, 0};
        for (int d = S - 1; d >= 1; --d) {
            uint32_t w = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int t = src[d * plane + (jl4 * 4 + q) * kBM] + carry[q];
                w |= (uint32_t(t) & 255u) << (8 * q);
                carry[q] = (t + 128) >> 8;
            }
            reinterpret_cast<uint32_t*>(L)[((int64_t(kb) * (s_cap - 1) + (d - 1)) * (np / 4) + j0 / 4 + jl4) * mp + i] = w;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            T[(int64_t(kb) * np + j0 + jl4 * 4 + q) * mp + i] = src[(jl4 * 4 + q) * kBM] + carry[q];
    }
}

// Per-tile mode: the order in which the tiles of C are dealt to the workgroups.  An XCD runs its tiles in
// rounds of 32 that keep in step to share panels in L2; a round that mixes tiles of different slice counts
// falls out of step when its light tiles finish (their successors wait in vain for the heavy ones and then
// run alone: measured 18.0 ms instead of 13.9 ms for 64 ten-slice tiles lying in one block column).  So the
// tiles are sorted by slice count, heaviest first and otherwise in the usual block order, and the sorted
// groups of 32 are dealt to the XCDs in turn: group g is round g / 8 of XCD g % 8.  Rounds are then uniform
// but for one per slice count, the heavy rounds are spread over the XCDs, and the lightest tiles end up in
// the partial last round or the k-split launch.  `first` = tiles of the first launch (its XCD ranges are what
// the groups are dealt into), of which the leading first / 256 * 256 sorted tiles are dealt; the others keep
// the sorted order in the positions that remain.  order[position] = index of the tile in the block order.
// One workgroup; a stable counting sort over the slice counts 0 .. kMaxSlices.
__global__ __launch_bounds__(256) void tile_order_kernel(const int32_t* __restrict__ tile_S, int32_t* __restrict__ order,
                                                         int nti, int ntj, int first, int deal, const Record* rec) {
    if (rec->res.fallback) return;
    const int tiles = nti * ntj, tid = threadIdx.x;
    if (!deal) {
        for (int lin = tid; lin < tiles; lin += 256) order[lin] = lin;
        return;
    }
    __shared__ int cnt[kMaxSlices + 1][256];
    __shared__ int base[kMaxSlices + 1];
    const int chunk = (tiles + 255) / 256;
    const int lo = min(tiles, tid * chunk), hi = min(tiles, lo + chunk);
    auto key_of = [&](int lin) -> int {
        int ti, tj;
        lin_to_tile(lin, nti, ntj, ti, tj);
        return min(max(tile_S[tj * nti + ti], 0), kMaxSlices);
    };
    for (int k = 0; k <= kMaxSlices; ++k) cnt[k][tid] = 0;
    for (int lin = lo; lin < hi; ++lin) ++cnt[key_of(lin)][tid];
    __syncthreads();
    if (tid <= kMaxSlices) {      // exclusive prefix over the threads' chunks, per key
        int run = 0;
        for (int t = 0; t < 256; ++t) {
            const int c = cnt[tid][t];
            cnt[tid][t] = run;
            run += c;
        }
        base[tid] = run;
    }
    __syncthreads();
    if (tid == 0) {               // keys in descending order
        int run = 0;
        for (int k = kMaxSlices; k >= 0; --k) {
            const int c = base[k];
            base[k] = run;
            run += c;
        }
    }
    __syncthreads();
    const int per = first >> 3, rem = first & 7, rounds = first / (8 * kRoundTiles), dealt = rounds * 8 * kRoundTiles;
    for (int lin = lo; lin < hi; ++lin) {
        const int k = key_of(lin);
        const int si = base[k] + cnt[k][tid]++;      // position in the sorted sequence
        int q = si;
        if (si < dealt) {
            const int g = si / kRoundTiles, wpos = si % kRoundTiles, r = g >> 3, x = g & 7;
            q = x * per + min(x, rem) + r * kRoundTiles + wpos;
        } else if (si < first) {
            // what is left of the XCD ranges behind their dealt rounds, XCD by XCD
            int t = si - dealt;
            for (int x = 0; x < 8; ++x) {
                const int left = per + (x < rem ? 1 : 0) - rounds * kRoundTiles;
                if (t < left) {
                    q = x * per + min(x, rem) + rounds * kRoundTiles + t;
                    break;
                }
                t -= left;
            }
        }
        order[q] = lin;
    }
}

void launch_gemm_i8(hipStream_t st, const Workspace& w, const Problem& p) {
    // the attribute is per device and cheap to set; no process-wide cache that a second device would miss
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_i8_kernel<false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_i8_kernel<true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
    const int nti = int(p.mp / kBM), ntj = int(p.np / kBN);
    const int tiles = nti * ntj;
    const int64_t kt_total = p.kp / kBK;
    const int planes = p.nkb * p.s_cap;
    const int32_t* tile_S = p.tile_mode ? w.tile_S : nullptr;
    // the workgroup-to-XCD reasoning behind the in-step waits holds for the whole chip only
    // (8 XCDs of 32 CUs); a partitioned device runs the same kernel without them
    const int full_chip = p.num_cu == 8 * kRoundTiles ? 1 : 0;
    // k split for `count` tiles that cannot fill the chip: about one workgroup per CU, each part
    // keeping at least kMinSplitSteps K steps; the parts add into the raw buffer with integer atomics
    auto split_for = [&](int count) -> int {
        int zs = p.num_cu / count;
        if (zs > kt_total / kMinSplitSteps) zs = int(kt_total / kMinSplitSteps);
        if (count > p.raw_slots) zs = 1;      // cannot happen: a split launch has fewer tiles than CUs
        return zs < 1 ? 1 : zs;
    };
    auto launch = [&](int begin, int count, int zs) {
        if (zs > 1)
            hipLaunchKernelGGL(zero_raw_kernel, dim3(unsigned(count), unsigned(planes)), dim3(256), 0, st, w.raw,
                               p.raw_slots, w.rec);
        if (zs > 1)
            hipLaunchKernelGGL(gemm_i8_kernel<true>, dim3(unsigned(count) * unsigned(zs)), dim3(256), kGemmLds, st,
                               w.As, w.Bs, w.T, w.L, w.raw, p.raw_slots, p.mp, p.np, p.kp, p.s_cap, w.rec, full_chip,
                               zs, begin, count, tile_S);
        else
            hipLaunchKernelGGL(gemm_i8_kernel<false>, dim3(unsigned(count)), dim3(256), kGemmLds, st, w.As, w.Bs,
                               w.T, w.L, w.raw, p.raw_slots, p.mp, p.np, p.kp, p.s_cap, w.rec, full_chip, 1, begin,
                               count, tile_S);
        if (zs > 1)
            hipLaunchKernelGGL(aggregate_raw_kernel, dim3(unsigned(count), unsigned(p.nkb)), dim3(256), 0, st, w.raw,
                               p.raw_slots, w.T, w.L, p.mp, p.np, p.kp, p.s_cap, nti, ntj, begin, w.rec, tile_S);
    };
    // Tiles are dealt in rounds of one per CU.  A call with less than three quarters of a round is
    // split along k as a whole; otherwise the full rounds run unsplit and a last round that would
    // be less than three quarters full is split along k in a launch of its own.
    const int round = p.num_cu;
    const int full = tiles / round * round, rest = tiles - full;
    if (p.tile_mode) {
        const bool two_launches = full != 0 && rest != 0 && rest * 4 <= round * 3 && split_for(rest) != 1;
        const int first = two_launches ? full : tiles;
        const int deal = (full_chip && full != 0 && tiles <= (1 << 16)) ? 1 : 0;
        hipLaunchKernelGGL(tile_order_kernel, dim3(1), dim3(256), 0, st, w.tile_S, w.tile_S + tiles, nti, ntj, first, deal,
                           w.rec);
    }
    if (full == 0) {
        launch(0, tiles, rest * 4 <= round * 3 ? split_for(tiles) : 1);
    } else if (rest == 0 || rest * 4 > round * 3 || split_for(rest) == 1) {
        launch(0, tiles, 1);
    } else {
        launch(0, full, 1);
        launch(full, rest, split_for(rest));
    }
}

}  // namespace oz
