// Coarsened Exponent Span Capacity and the verdict.
// (paper: section "ESC", formula ESC = exp(x_p) + exp(y_q) - exp(z_r) maximised over the mn dot
//  products with z_r estimated from per-block Max/Min exponents, plus the +1 safety margin;
//  sections "Heuristic run time Selection" and "GPU-Resident Integration" for the verdict.)
//
// The estimate is a max-plus matrix product  zt = U (x) V  with inner length 2G:
//   zt_ij = max_h ( U[h][i] + V[h][j] ),  U = [Max(xb); Min(xb)],  V = [Min(yb); Max(yb)],
// followed by  span = max_ij ( eA_i + eB_j - zt_ij ).  There is no matrix-unit form of max-plus
// on gfx950, so it runs on the vector ALU with packed int16 add/max: one lane instruction
// updates two (i,j) pairs.  Bound: plain ALU; 2 packed ops per h per two pairs.
#include "oz_internal.h"

namespace oz {

typedef short short2_t __attribute__((ext_vector_type(2)));
typedef short short8_t __attribute__((ext_vector_type(8)));

constexpr int kEscTile = 128;   // (i,j) tile per workgroup, 16x16 threads of 8x8 pairs
constexpr int kEscHChunk = 32;  // inner steps staged in LDS at a time
constexpr short kEscPadValue = -16384;  // two of them add to the int16 minimum without wrapping

__global__ __launch_bounds__(256) void esc_kernel(const int16_t* __restrict__ U,
                                                  const int16_t* __restrict__ V,
                                                  const int32_t* __restrict__ eA,
                                                  const int32_t* __restrict__ eB, int64_t mp,
                                                  int64_t np, int H2, Record* rec) {
    __shared__ short8_t Ut[kEscHChunk][kEscTile / 8];
    __shared__ short8_t Vt[kEscHChunk][kEscTile / 8];
    if (rec->infnan) return;   // Inf/NaN already forces the native path; skip the O(mnk/b) work

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
    if ((threadIdx.x & 63) == 0 && best > 0) atomicMax(&rec->span_max, best);
}

// One thread: slice count and fallback decision from the scan flag and the ESC.
__global__ void verdict_kernel(Record* rec, oz_opts_t o, oz_heuristic_t hm, int kind,
                               int64_t m, int64_t n, int64_t k, int s_cap,
                               oz_result_t* user_result) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    oz_result_t r;
    r.fallback = 0; r.reason = 0; r.slices_used = 0; r.esc = -1; r.required_bits = 0; r.infnan = 0;
    if (kind == 2) {   // nothing to multiply (k == 0 or alpha == 0)
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
        if (o.mode == OZ_FORCED_GUARDED) {
            r.slices_used = s_fixed;
        } else if (r.required_bits > o.max_bits) {
            r.fallback = 1; r.reason = 2;
        } else if (o.mode == OZ_FIXED_GUARDED) {
            r.slices_used = s_fixed;
        } else {
            int S = (o.target_bits + esc + 1 + kHeadroomBits + 7) / 8;
            S = max(1, min(S, kMaxSlices));
            bool slower = false;
            if (o.heuristic) {
                const int64_t flops = 2 * m * n * k;
                const int64_t pairs = int64_t(S) * (S + 1) / 2;
                const int64_t stream = (8 + S) * (m * k + k * n) + (8 * int64_t(S) + 16) * m * n;
                const int64_t t_emu = hm.fixed_ns + (flops / hm.int8_ops_per_ns) * pairs + stream / hm.bytes_per_ns;
                const int64_t t_f64 = flops / hm.fp64_flops_per_ns;
                slower = t_emu > t_f64;
            }
            if (slower) { r.fallback = 1; r.reason = 3; }
            else r.slices_used = S;
        }
    }
    // the workspace holds s_cap slice planes; the host sized it so that this never binds
    if (!r.fallback && r.slices_used > s_cap) r.slices_used = s_cap;
    rec->res = r;
    if (user_result) *user_result = r;
}

void launch_esc(hipStream_t st, const Workspace& w, const Problem& p) {
    hipLaunchKernelGGL(esc_kernel, dim3(unsigned(p.mp / kEscTile), unsigned(p.np / kEscTile)), dim3(256), 0,
                       st, w.U, w.V, w.eA, w.eB, p.mp, p.np, 2 * p.G, w.rec);
}

void launch_verdict(hipStream_t st, const Workspace& w, const Problem& p, const oz_opts_t& o,
                    const oz_heuristic_t& hm, int kind, oz_result_t* user_result) {
    hipLaunchKernelGGL(verdict_kernel, dim3(1), dim3(64), 0, st, w.rec, o, hm, kind, p.m, p.n,
                       p.k, p.s_cap, user_result);
}

}  // namespace oz
