// Coarsened Exponent Span Capacity and the verdict.
// (paper: section "ESC", formula ESC = exp(x_p) + exp(y_q) - exp(z_r) maximised over the mn dot
//  products with z_r estimated from per-block Max/Min exponents, plus the +1 safety margin;
//  sections "Heuristic run time Selection" and "GPU-Resident Integration" for the verdict.)
//
// The estimate is a max-plus matrix product  zt = U (x) V  with inner length 2G:
//   zt_ij = max_h ( U[h][i] + V[h][j] ),  U = [Max(xb); Min(xb)],  V = [Min(yb); Max(yb)],
// followed by  span = max_ij ( eA_i + eB_j - zt_ij ).
//
// Two kernels compute it.
//  * esc_mfma_kernel (always runs): the max-plus product mapped onto the BF16 matrix unit.
//    With u = U[h][i] - eA_i <= 0 and v = V[h][j] - eB_j <= 0 the table entries are encoded as
//    the powers of two 2^(5u+61) and 2^(5v+61) (exact in BF16; entries below -37 and the "zero"
//    sentinels become 0).  One MFMA sums 16 such products in FP32; all terms are non-negative, so
//    2^(5t+122) <= sum <= 16 * 2^(5t+122) with t = max_h (u+v) over the 16 steps, whatever the
//    order and rounding of the accumulation, and floor((exponent(sum) - 122) / 5) = t exactly.
//    The running maximum over the chunks of 16 is kept on the raw FP32 bit patterns.  A pair
//    whose result is below -37 (or has no candidate at all) may have lost candidates to the
//    clamping, so it raises rec->esc_exact instead of contributing.
//  * esc_kernel (runs only when that flag is set): the same product on the vector ALU with packed
//    int16 add/max over the unencoded tables, one lane instruction per two (i,j) pairs.
// Both give the exact coarsened ESC; the first covers spans up to 37 bits at matrix-unit speed.
#include "oz_internal.h"

namespace oz {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kEncScale = 5;     // exponent units per bit of span; 16 equal terms stay below 2^5
constexpr int kEncBias = 61;     // 2*61 + 4 < 128: a chunk sum cannot overflow FP32
constexpr int kEncRange = 37;    // 5*(-37) + 61 >= -126: smallest encodable entry (BF16 normal)
constexpr int kEncChunk = 16;    // inner steps per MFMA (K of v_mfma_f32_32x32x16_bf16)

// enc[(h/8) * rows_p + r][h%8] = BF16 bits of 2^(5*(tab[h][r] - e[r]) + 61), or 0
__global__ __launch_bounds__(256) void esc_encode_kernel(const int16_t* __restrict__ tab,
                                                         const int32_t* __restrict__ e,
                                                         int64_t rows_p, int H2,
                                                         uint4* __restrict__ enc) {
    const int64_t r = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int hc = blockIdx.y;
    const int er = e[r];
    uint32_t w[4];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int h = hc * 8 + q;
        uint32_t bits = 0;
        if (h < H2) {
            const int x = tab[int64_t(h) * rows_p + r];
            const int d = x - er;
            if (x > kSumRealFloor / 2 && d >= -kEncRange && d <= 0)
                bits = uint32_t(kEncScale * d + kEncBias + 127) << 7;
        }
        if (q & 1) w[q >> 1] |= bits << 16; else w[q >> 1] = bits;
    }
    enc[int64_t(hc) * rows_p + r] = make_uint4(w[0], w[1], w[2], w[3]);
}

// grid (mp/128, np/128); 4 waves of 64x64 pairs, 2x2 MFMA tiles of 32x32 each.
__global__ __launch_bounds__(256) void esc_mfma_kernel(const uint4* __restrict__ EU,
                                                       const uint4* __restrict__ EV, int64_t m,
                                                       int64_t n, int64_t mp, int64_t np,
                                                       int steps, Record* rec,
                                                       int32_t* __restrict__ tile_span) {
    if (rec->infnan) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane & 31, lh = lane >> 5;
    const int64_t i0 = int64_t(blockIdx.x) * 128 + (wave & 1) * 64;
    const int64_t j0 = int64_t(blockIdx.y) * 128 + (wave >> 1) * 64;
    const uint4* pa = EU + int64_t(lh) * mp + i0 + lr;
    const uint4* pb = EV + int64_t(lh) * np + j0 + lr;

    uint32_t run[2][2][16];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) run[a][b][r] = 0;

    const f32x16_t zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    // Two chunks per step (the tables are zero-padded to a multiple of 32 inner steps).  The
    // operands of the next step are requested before the current step's arithmetic; the loads are
    // written as asm so that they stay where they are issued, and the explicit wait ties the
    // destination registers to the point where the data has arrived.
    u32x4_t X[8], Y[8];
    int loaded = 0;   // step the pointers address
#define OZ_ESC_ISSUE(buf)                                                                      \
    do {                                                                                       \
        const uint4* pa1_ = pa + 2 * mp;                                                       \
        const uint4* pb1_ = pb + 2 * np;                                                       \
        asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(buf[0]) : "v"(pa));             \
        asm volatile("global_load_dwordx4 %0, %1, off offset:512" : "=&v"(buf[1]) : "v"(pa));  \
        asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(buf[2]) : "v"(pa1_));           \
        asm volatile("global_load_dwordx4 %0, %1, off offset:512" : "=&v"(buf[3]) : "v"(pa1_));\
        asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(buf[4]) : "v"(pb));             \
        asm volatile("global_load_dwordx4 %0, %1, off offset:512" : "=&v"(buf[5]) : "v"(pb));  \
        asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(buf[6]) : "v"(pb1_));           \
        asm volatile("global_load_dwordx4 %0, %1, off offset:512" : "=&v"(buf[7]) : "v"(pb1_));\
        if (loaded + 1 < steps) { pa += 4 * mp; pb += 4 * np; ++loaded; }  /* else: re-read */   \
        __builtin_amdgcn_sched_barrier(0);   /* the arithmetic below must not move above the loads */ \
    } while (0)
#define OZ_ESC_WAIT(buf)                                                                       \
    __builtin_amdgcn_sched_barrier(0);       /* the arithmetic above stays above the wait */   \
    asm volatile("s_waitcnt vmcnt(0)"                                                          \
                 : "+v"(buf[0]), "+v"(buf[1]), "+v"(buf[2]), "+v"(buf[3]), "+v"(buf[4]),       \
                   "+v"(buf[5]), "+v"(buf[6]), "+v"(buf[7]));                                  \
    __builtin_amdgcn_sched_barrier(0)
#define OZ_ESC_COMPUTE(buf)                                                                    \
    _Pragma("unroll") for (int a = 0; a < 2; ++a) _Pragma("unroll") for (int b = 0; b < 2; ++b) { \
        const u32x16_t d0 = __builtin_bit_cast(u32x16_t, __builtin_amdgcn_mfma_f32_32x32x16_bf16( \
            __builtin_bit_cast(bf16x8_t, buf[a]), __builtin_bit_cast(bf16x8_t, buf[4 + b]), zero, 0, 0, 0)); \
        const u32x16_t d1 = __builtin_bit_cast(u32x16_t, __builtin_amdgcn_mfma_f32_32x32x16_bf16( \
            __builtin_bit_cast(bf16x8_t, buf[2 + a]), __builtin_bit_cast(bf16x8_t, buf[6 + b]), zero, 0, 0, 0)); \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) /* sums are >= 0: unsigned order is numeric order */ \
            run[a][b][r] = max(run[a][b][r], max(d0[r], d1[r]));                                \
    }

    OZ_ESC_ISSUE(X);
    for (int c = 0; c < steps; c += 2) {
        OZ_ESC_WAIT(X);
        OZ_ESC_ISSUE(Y);
        OZ_ESC_COMPUTE(X);
        OZ_ESC_WAIT(Y);
        OZ_ESC_ISSUE(X);
        if (c + 1 < steps) { OZ_ESC_COMPUTE(Y); }
    }
    OZ_ESC_WAIT(X);   // nothing may be in flight when the wave ends
#undef OZ_ESC_ISSUE
#undef OZ_ESC_WAIT
#undef OZ_ESC_COMPUTE

    // The span of a pair decreases with its sum, so the largest span of the tile belongs to the
    // smallest sum: reduce the raw bit patterns first, convert once.
    uint32_t least = 0xFFFFFFFFu;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t i = i0 + a * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const int64_t j = j0 + b * 32 + lr;
                if (i < m && j < n) least = min(least, run[a][b][r]);
            }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) least = min(least, uint32_t(__shfl_xor(int(least), off)));
    __shared__ uint32_t wave_least[4];
    if (lane == 0) wave_least[wave] = least;
    __syncthreads();
    if (threadIdx.x != 0) return;
    least = min(min(wave_least[0], wave_least[1]), min(wave_least[2], wave_least[3]));
    if (least == 0xFFFFFFFFu) return;               // the tile holds padding only
    // exponent(sum) - 122 lies in [5t, 5t+4]; shifted by 5*64 so that the division is of a
    // non-negative number
    const int E = int(least >> 23) - 127 - 2 * kEncBias;
    const int t = (E + kEncScale * 64) / kEncScale - 64;
    if (t < -kEncRange) {
        // Below the encodable range (or no candidate at all): the int16 kernel visits every pair,
        // including the ones this tile resolved, so nothing else needs to be recorded here.
        atomicOr(&rec->esc_exact, 1);
    } else {
        // this 128 x 128 block is resolved exactly: its largest span goes to the C block it lies in
        // (four such blocks per kTile x kTile block) and to the global maximum
        atomicMax(&tile_span[(blockIdx.y >> 1) * (mp / kTile) + (blockIdx.x >> 1)], -t);
        // a stale read only costs a redundant atomic; the maximum is monotone
        if (-t > *reinterpret_cast<volatile int32_t*>(&rec->span_max)) atomicMax(&rec->span_max, -t);
    }
}

typedef short short2_t __attribute__((ext_vector_type(2)));
typedef short short8_t __attribute__((ext_vector_type(8)));

constexpr int kEscTile = 128;   // (i,j) tile per workgroup, 16x16 threads of 8x8 pairs
constexpr int kEscHChunk = 32;  // inner steps staged in LDS at a time
constexpr short kEscPadValue = -16384;  // two of them add to the int16 minimum without wrapping

__global__ __launch_bounds__(256) void esc_kernel(const int16_t* __restrict__ U,
                                                  const int16_t* __restrict__ V,
                                                  const int32_t* __restrict__ eA,
                                                  const int32_t* __restrict__ eB, int64_t mp,
                                                  int64_t np, int H2, Record* rec,
                                                  int32_t* __restrict__ tile_span) {
    __shared__ short8_t Ut[kEscHChunk][kEscTile / 8];
    __shared__ short8_t Vt[kEscHChunk][kEscTile / 8];
    // Inf/NaN already forces the native path; otherwise run only for what the MFMA kernel left open
    if (rec->infnan || !rec->esc_exact) return;

    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t i0 = int64_t(blockIdx.x) * kEscTile, j0 = int64_t(blockIdx.y) * kEscTile;

    short2_t acc[8][4];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = short2_t{-32768, -32768};

    for (int h0 = 0; h0 < H2; h0 += kEscHChunk) {
        __syncthreads();
        // 32 x 128 int16 per table = 512 vectors of 8; two per thread
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int v = threadIdx.x + t * 256;
            const int hh = v >> 4, col = v & 15;
            short8_t uu, vv;
            if (h0 + hh < H2) {
                uu = *reinterpret_cast<const short8_t*>(U + int64_t(h0 + hh) * mp + i0 + col * 8);
                vv = *reinterpret_cast<const short8_t*>(V + int64_t(h0 + hh) * np + j0 + col * 8);
            } else {
                uu = short8_t(kEscPadValue);
                vv = short8_t(kEscPadValue);
            }
            Ut[hh][col] = uu;
            Vt[hh][col] = vv;
        }
        __syncthreads();
#pragma unroll 4
        for (int hh = 0; hh < kEscHChunk; ++hh) {
            const short8_t u = Ut[hh][ty];
            const short8_t v = Vt[hh][tx];
            const short2_t v2[4] = {short2_t{v[0], v[1]}, short2_t{v[2], v[3]},
                                    short2_t{v[4], v[5]}, short2_t{v[6], v[7]}};
#pragma unroll
            for (int a = 0; a < 8; ++a) {
                const short2_t ua = short2_t{u[a], u[a]};
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[a][c] = __builtin_elementwise_max(acc[a][c], ua + v2[c]);
            }
        }
    }

    int best = 0;
#pragma unroll
    for (int a = 0; a < 8; ++a) {
        const int ea = eA[i0 + ty * 8 + a];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int z = acc[a][c][q];
                const int eb = eB[j0 + tx * 8 + c * 2 + q];
                int span;
                if (z >= kSumRealFloor) span = ea + eb - z;          // a real exponent sum
                else if (z >= kSumDeadBelow) span = kEscCap;          // no candidate: unbounded
                else span = 0;                                        // identically zero product
                best = max(best, span);
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) best = max(best, __shfl_xor(best, off));
    if ((threadIdx.x & 63) == 0) {
        // this kernel visits every pair, so its block maxima complete the per-block table as well
        // (kEscTile x kEscTile blocks, four per kTile x kTile block of C)
        static_assert(kTile == 2 * kEscTile, "four ESC blocks per block of C");
        atomicMax(&tile_span[(blockIdx.y >> 1) * (mp / kTile) + (blockIdx.x >> 1)], best);
        // the maximum is monotone: a stale read only costs a redundant atomic
        if (best > *reinterpret_cast<volatile int32_t*>(&rec->span_max)) atomicMax(&rec->span_max, best);
    }
}

// Per-tile mode: slice count of every kTile x kTile block of C from the largest span inside it, plus
// the two sums the verdict needs (pair products over all blocks, smallest count).
__global__ __launch_bounds__(256) void tile_verdict_kernel(Record* rec, const int32_t* __restrict__ tile_span,
                                                           int32_t* __restrict__ tile_S, int64_t tiles,
                                                           int target_bits) {
    const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
    unsigned long long pairs = 0;
    int smin = kMaxSlices;
    if (t < tiles) {
        const int esc = min(tile_span[t] + 1, kEscCap);
        int S = (target_bits + esc + 1 + kHeadroomBits + 7) / 8;
        S = max(1, min(S, kMaxSlices));
        tile_S[t] = S;
        pairs = (unsigned long long)(S) * (S + 1) / 2;
        smin = S;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        pairs += __shfl_xor(pairs, off);
        smin = min(smin, __shfl_xor(smin, off));
    }
    if ((threadIdx.x & 63) == 0 && pairs) {
        atomicAdd(&rec->pair_acc, pairs);
        atomicMin(&rec->smin_acc, smin);
    }
}

// One thread: slice count and fallback decision from the scan flag and the ESC.
__global__ void verdict_kernel(Record* rec, oz_opts_t o, oz_heuristic_t hm, int kind,
                               int64_t m, int64_t n, int64_t k, int s_cap, int tile_mode,
                               oz_result_t* user_result) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    oz_result_t r;
    r.fallback = 0; r.reason = 0; r.slices_used = 0; r.esc = -1; r.required_bits = 0; r.infnan = 0;
    r.slices_min = 0; r.reserved_ = 0; r.pair_tiles = 0;
    const int64_t tiles = ((m + kTile - 1) / kTile) * ((n + kTile - 1) / kTile);
    bool per_tile = false;    // the blocks of C carry their own counts (tile_verdict_kernel ran)
    if (kind == 2 || kind == 3) {
        // 2: nothing to multiply (k == 0 or alpha == 0); 3: the host's cost model says that no slice
        // count this call could get beats the native GEMM, so nothing was scanned
        if (kind == 3) { r.fallback = 1; r.reason = 3; }
        rec->res = r;
        if (user_result) *user_result = r;
        return;
    }
    int s_fixed = o.slices > 0 ? o.slices : (o.max_bits + 1 + 7) / 8;
    s_fixed = max(1, min(s_fixed, kMaxSlices));
    if (o.mode == OZ_NATIVE) {
        r.fallback = 1; r.reason = 4;
    } else if (o.mode == OZ_FIXED_UNGUARDED) {
        r.slices_used = s_fixed;
    } else if (rec->infnan) {
        r.fallback = 1; r.reason = 1; r.infnan = 1;
    } else {
        const int esc = min(rec->span_max + 1, kEscCap);
        r.esc = esc;
        r.required_bits = o.target_bits + esc;
        // slices that hold required_bits, the sign and the headroom bit
        int S = (o.target_bits + esc + 1 + kHeadroomBits + 7) / 8;
        if (o.mode == OZ_FORCED_GUARDED) {
            r.slices_used = s_fixed;
        } else if (r.required_bits > o.max_bits) {
            r.fallback = 1; r.reason = 2;
        } else if (o.mode == OZ_FIXED_GUARDED) {
            // the fixed slices must really carry the bits (S slices carry 8S - 2: "55 bits" is 54)
            if (S > s_fixed) { r.fallback = 1; r.reason = 2; }
            else r.slices_used = s_fixed;
        } else {
            S = max(1, min(S, kMaxSlices));
            per_tile = tile_mode != 0;
            bool slower = false;
            if (o.heuristic) {
                const int64_t flops = 2 * m * n * k;
                // pair products per block of C: S(S+1)/2, or the mean over the blocks, rounded up
                const int64_t pairs = per_tile ? int64_t((rec->pair_acc + (unsigned long long)(tiles) - 1) /
                                                         (unsigned long long)(tiles))
                                               : int64_t(S) * (S + 1) / 2;
                const int64_t stream = (16 + S) * (m * k + k * n) + (2 * int64_t(S) + 22) * m * n;
                const int64_t t_emu = hm.fixed_ns + (flops / hm.int8_ops_per_ns) * pairs + stream / hm.bytes_per_ns;
                const int64_t t_f64 = flops / hm.fp64_flops_per_ns;
                slower = t_emu > t_f64;
            }
            if (slower) { r.fallback = 1; r.reason = 3; }
            else r.slices_used = S;
        }
    }
    // The workspace holds s_cap slice planes and the host sized it for the largest count these options
    // can select, so this never binds; if it ever did, running with fewer slices would lose bits
    // silently, so the call goes native and says why.
    if (!r.fallback && r.slices_used > s_cap) { r.fallback = 1; r.reason = 2; r.slices_used = 0; }
    if (!r.fallback && r.slices_used > 0) {
        r.slices_min = per_tile ? rec->smin_acc : r.slices_used;
        r.pair_tiles = per_tile ? int64_t(rec->pair_acc) : tiles * (int64_t(r.slices_used) * (r.slices_used + 1) / 2);
    }
    rec->res = r;
    if (user_result) *user_result = r;
}

void launch_esc(hipStream_t st, const Workspace& w, const Problem& p) {
    const int H2 = 2 * p.G;
    const int steps = (H2 + 2 * kEncChunk - 1) / (2 * kEncChunk);   // 32 inner steps (4 groups of 8) each
    hipLaunchKernelGGL(esc_encode_kernel, dim3(unsigned(p.mp / 256), unsigned(steps * 4)), dim3(256), 0, st,
                       w.U, w.eA, p.mp, H2, reinterpret_cast<uint4*>(w.EU));
    hipLaunchKernelGGL(esc_encode_kernel, dim3(unsigned(p.np / 256), unsigned(steps * 4)), dim3(256), 0, st,
                       w.V, w.eB, p.np, H2, reinterpret_cast<uint4*>(w.EV));
    hipLaunchKernelGGL(esc_mfma_kernel, dim3(unsigned(p.mp / 128), unsigned(p.np / 128)), dim3(256), 0, st,
                       reinterpret_cast<const uint4*>(w.EU), reinterpret_cast<const uint4*>(w.EV), p.m, p.n,
                       p.mp, p.np, steps, w.rec, w.tile_span);
    hipLaunchKernelGGL(esc_kernel, dim3(unsigned(p.mp / kEscTile), unsigned(p.np / kEscTile)), dim3(256), 0,
                       st, w.U, w.V, w.eA, w.eB, p.mp, p.np, 2 * p.G, w.rec, w.tile_span);
}

void launch_tile_verdict(hipStream_t st, const Workspace& w, const Problem& p, const oz_opts_t& o) {
    const int64_t tiles = (p.mp / kTile) * (p.np / kTile);
    hipLaunchKernelGGL(tile_verdict_kernel, dim3(unsigned((tiles + 255) / 256)), dim3(256), 0, st, w.rec,
                       w.tile_span, w.tile_S, tiles, o.target_bits);
}

void launch_verdict(hipStream_t st, const Workspace& w, const Problem& p, const oz_opts_t& o,
                    const oz_heuristic_t& hm, int kind, oz_result_t* user_result) {
    hipLaunchKernelGGL(verdict_kernel, dim3(1), dim3(64), 0, st, w.rec, o, hm, kind, p.m, p.n,
                       p.k, p.s_cap, p.tile_mode, user_result);
}

}  // namespace oz
