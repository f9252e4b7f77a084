// Slice-pair INT8 GEMMs with exact int32 accumulation: the one dense contraction of the method.
// (paper: section "FP64 Emulation on Low-Precision Units": products are computed slice by slice;
//  section "ESC": cost is quadratic in the slice count; the kept pairs are s + t <= S - 1, the
//  count behind "seven slices rather than eight: 22 % less compute"; section "Pre-processing
//  and Safety Checks": partial results are aggregated so that accumulators cannot overflow.)
//
//   P[kb][d][j][i] = sum_{s+t=d} sum_{l in k-block kb} As[s][i][l] * Bs[t][j][l],   d = 0..S-1
//
// One launch covers all S(S+1)/2 pairs: a workgroup owns a 256x256 tile of C and walks the
// anti-diagonals d; all pairs of one d accumulate into the same int32 registers (their k
// ranges are simply concatenated), so only S tiles are written per k-block.
//
// Mapping to gfx950: v_mfma_i32_32x32x32_i8, 4 waves per workgroup, each wave a 128x128
// sub-tile (4x4 MFMA tiles, 256 accumulator registers per lane).  K tile 128, LDS double
// buffered (2 x 64 KB of the CU's 160 KB).  The slice panels are stored [k/16][row][16], so a
// tile is a set of contiguous 4 KB runs in HBM and the LDS image [k chunk][row][16 B] is read
// by the MFMA operand loads (one ds_read_b128 per lane: row = lane%32, k chunk = lane/32)
// without bank conflicts.  The B-slices feed the MFMA's row operand and the A-slices its column
// operand, so the lane index of the result runs along i and stores to P (i contiguous) coalesce.
// Workgroup ids are remapped so that the tiles resident on one XCD form a compact block and
// share their A and B panels in that XCD's L2.
#include "oz_internal.h"

namespace oz {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBM = 256;             // tile extent along i (rows of op(A))
constexpr int kBN = 256;             // tile extent along j (columns of op(B))
constexpr int kBK = kKPad;           // 128
constexpr int kStageBytes = (kBM + kBN) * kBK;   // 64 KB
constexpr int kGemmLds = 2 * kStageBytes;

__device__ __forceinline__ v4i as_v4i(const uint4& v) { return v4i{int(v.x), int(v.y), int(v.z), int(v.w)}; }

// linear workgroup id -> tile coordinates.  Ids are dealt round-robin to the 8 XCDs by the
// hardware; each XCD is given a contiguous range of a tile order in which 32 consecutive tiles
// form a 4 (i) x 8 (j) block.
__device__ __forceinline__ void tile_of(int bid, int nti, int ntj, int& ti, int& tj) {
    const int total = nti * ntj;
    const int xcd = bid & 7, slot = bid >> 3;
    const int per = total >> 3, rem = total & 7;
    const int lin = xcd * per + min(xcd, rem) + slot;
    constexpr int GW = 8;
    const int panel = lin / (GW * nti);
    const int in_panel = lin - panel * GW * nti;
    const int w = min(GW, ntj - panel * GW);
    ti = in_panel / w;
    tj = panel * GW + in_panel % w;
}

__global__ __launch_bounds__(256) void gemm_i8_kernel(const int8_t* __restrict__ As,
                                                      const int8_t* __restrict__ Bs,
                                                      int32_t* __restrict__ P, int64_t mp,
                                                      int64_t np, int64_t kp, int s_cap,
                                                      const Record* rec) {
    extern __shared__ __align__(16) uint8_t lds[];
    if (rec->res.fallback) return;
    const int S = rec->res.slices_used;
    // k-range one int32 accumulator can take with S slices (S*kblk digit products of at most 2^14)
    const int64_t kblk = ((int64_t(1) << 17) - 1) / S / 256 * 256;
    const int nkb = int((kp + kblk - 1) / kblk);

    int ti, tj;
    tile_of(blockIdx.x, int(mp / kBM), int(np / kBN), ti, tj);
    const int64_t i0 = int64_t(ti) * kBM, j0 = int64_t(tj) * kBN;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wi = wave & 1, wj = wave >> 1;

    v16i acc[4][4];   // [fj][fi]
    const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = zero;

    auto kt_count = [&](int kb) -> int {
        const int64_t k0 = int64_t(kb) * kblk;
        const int64_t k1 = (k0 + kblk < kp) ? k0 + kblk : kp;
        return int((k1 - k0) / kBK);
    };

    // (nkb_, nd, ns, nkt) walks the (k-block, anti-diagonal, pair, K step) sequence one tile
    // ahead of the compute, so the prefetch runs across pair and anti-diagonal boundaries
    // without a bubble.  After the last tile it stays put (the final prefetch is discarded).
    int nkb_ = 0, nd = 0, ns = 0, nkt = 0;
    int nxt_ktc = kt_count(0);
    const uint4* gA = reinterpret_cast<const uint4*>(As) + i0 + threadIdx.x;
    const uint4* gB = reinterpret_cast<const uint4*>(Bs) + j0 + threadIdx.x;
    const int64_t planeA = (kp / 16) * mp, planeB = (kp / 16) * np;   // uint4 per slice plane

    // The prefetch is issued with inline assembly: a plain C++ load from read-only memory is moved
    // by the compiler down to its use (the LDS store after the MFMA block), which would expose the
    // whole memory latency.  The compiler does not count these loads, so OZ_WAIT_PREFETCH() waits
    // for them explicitly and ties the staging registers to the wait.
    v4i sa[kBK / 16], sb[kBK / 16];
#define OZ_PREFETCH()                                                                        \
    {                                                                                        \
        const int64_t kc = (int64_t(nkb_) * kblk) / 16 + int64_t(nkt) * (kBK / 16);          \
        const uint4* pa = gA + int64_t(ns) * planeA + kc * mp;                               \
        const uint4* pb = gB + int64_t(nd - ns) * planeB + kc * np;                          \
        _Pragma("unroll") for (int q = 0; q < kBK / 16; ++q) {                               \
            asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(sa[q]) : "v"(pa + q * mp)); \
            asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(sb[q]) : "v"(pb + q * np)); \
        }                                                                                    \
    }
#define OZ_ADVANCE()                                                                         \
    {                                                                                        \
        if (++nkt == nxt_ktc) {                                                              \
            nkt = 0;                                                                         \
            if (++ns > nd) {                                                                 \
                ns = 0;                                                                      \
                if (++nd == S) {                                                             \
                    nd = 0;                                                                  \
                    if (++nkb_ == nkb) nkb_ = nkb - 1;                                       \
                    nxt_ktc = kt_count(nkb_);                                                \
                }                                                                            \
            }                                                                                \
        }                                                                                    \
    }
#define OZ_WAIT_PREFETCH()                                                                   \
    asm volatile("s_waitcnt vmcnt(0)"                                                        \
                 : "+v"(sa[0]), "+v"(sa[1]), "+v"(sa[2]), "+v"(sa[3]), "+v"(sa[4]), "+v"(sa[5]), \
                   "+v"(sa[6]), "+v"(sa[7]), "+v"(sb[0]), "+v"(sb[1]), "+v"(sb[2]), "+v"(sb[3]), \
                   "+v"(sb[4]), "+v"(sb[5]), "+v"(sb[6]), "+v"(sb[7]))
#define OZ_STAGE_TO_LDS(stage)                                                               \
    {                                                                                        \
        v4i* wa = reinterpret_cast<v4i*>(lds + (stage) * kStageBytes) + threadIdx.x;         \
        v4i* wb = reinterpret_cast<v4i*>(lds + (stage) * kStageBytes + kBM * kBK) + threadIdx.x; \
        _Pragma("unroll") for (int q = 0; q < kBK / 16; ++q) {                               \
            wa[q * kBM] = sa[q];                                                             \
            wb[q * kBN] = sb[q];                                                             \
        }                                                                                    \
    }

    static_assert(kBK / 16 == 8, "OZ_WAIT_PREFETCH lists 8 + 8 staging registers");
    OZ_PREFETCH();
    OZ_ADVANCE();
    OZ_WAIT_PREFETCH();
    OZ_STAGE_TO_LDS(0);
    __syncthreads();

    int buf = 0;
    for (int kb = 0; kb < nkb; ++kb) {
        const int ktc = kt_count(kb);
        for (int d = 0; d < S; ++d) {
            const int n_iter = (d + 1) * ktc;
            for (int it = 0; it < n_iter; ++it) {
                OZ_PREFETCH();
                __builtin_amdgcn_sched_barrier(0);

                const uint4* la = reinterpret_cast<const uint4*>(lds + buf * kStageBytes) + wi * 128 +
                                  (lane & 31) + (lane >> 5) * kBM;
                const uint4* lb = reinterpret_cast<const uint4*>(lds + buf * kStageBytes + kBM * kBK) +
                                  wj * 128 + (lane & 31) + (lane >> 5) * kBN;
                // operand fragments are double buffered in registers: the LDS reads of K sub-step
                // kk+1 are issued before the 16 MFMAs of sub-step kk
                v4i fa[2][4], fb[2][4];
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    fa[0][f] = as_v4i(la[f * 32]);
                    fb[0][f] = as_v4i(lb[f * 32]);
                }
#pragma unroll
                for (int kk = 0; kk < kBK / 32; ++kk) {
                    if (kk + 1 < kBK / 32) {
#pragma unroll
                        for (int f = 0; f < 4; ++f) {
                            fa[(kk + 1) & 1][f] = as_v4i(la[(kk + 1) * 2 * kBM + f * 32]);
                            fb[(kk + 1) & 1][f] = as_v4i(lb[(kk + 1) * 2 * kBN + f * 32]);
                        }
                    }
#pragma unroll
                    for (int fj = 0; fj < 4; ++fj)
#pragma unroll
                        for (int fi = 0; fi < 4; ++fi)
                            acc[fj][fi] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                                fb[kk & 1][fj], fa[kk & 1][fi], acc[fj][fi], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }

                // unconditional: after the last tile this rewrites a stage nobody reads again
                OZ_WAIT_PREFETCH();
                OZ_STAGE_TO_LDS(buf ^ 1);
                OZ_ADVANCE();
                __syncthreads();
                buf ^= 1;
            }

            // anti-diagonal d of k-block kb is complete: write the tile and restart from zero.
            // result register r of MFMA tile (fj, fi): j = fj*32 + 8*(r/4) + 4*(lane/32) + r%4,
            // i = fi*32 + lane%32
            int32_t* dst = P + ((int64_t(kb) * s_cap + d) * np + j0 + wj * 128) * mp + i0 + wi * 128;
#pragma unroll
            for (int fj = 0; fj < 4; ++fj)
#pragma unroll
                for (int fi = 0; fi < 4; ++fi) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int jl = fj * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                        const int il = fi * 32 + (lane & 31);
                        dst[int64_t(jl) * mp + il] = acc[fj][fi][r];
                    }
                    acc[fj][fi] = zero;
                }
        }
    }
}

#undef OZ_PREFETCH
#undef OZ_ADVANCE
#undef OZ_WAIT_PREFETCH
#undef OZ_STAGE_TO_LDS

void launch_gemm_i8(hipStream_t st, const Workspace& w, const Problem& p) {
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_i8_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds);
        attr_set = true;
    }
    const unsigned tiles = unsigned((p.mp / kBM) * (p.np / kBN));
    hipLaunchKernelGGL(gemm_i8_kernel, dim3(tiles), dim3(256), kGemmLds, st, w.As, w.Bs, w.P, p.mp, p.np,
                       p.kp, p.s_cap, w.rec);
}

}  // namespace oz
