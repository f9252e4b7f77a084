// FP64 recomposition of the integer anti-diagonal sums and the alpha/beta update.
// (paper: section "FP64 Emulation on Low-Precision Units": slice products are recombined;
//  section "Pre-processing and Safety Checks", second half: partial results are aggregated
//  before the terminal conversion to FP64, so an Inf can only appear in that last step.)
//
//   AB_ij = 2^(eA_i + eB_j - 10) * sum_kb sum_d 256^-d P[kb][d][j][i]
//   C_ij  = alpha * AB_ij + beta * C_ij           (C not read when beta == 0)
//
// Order (fixed, so results are reproducible): k-blocks ascending; inside a k-block Horner from
// the least significant anti-diagonal, R <- P_d + R * 2^-8; block results added unscaled; the
// power of two applied last with ldexp; alpha*AB and beta*C rounded separately, then added.
// HBM-bound: 4*S*nkb bytes read and 8 (+8 when beta != 0) bytes moved per element of C.
#include "oz_internal.h"

namespace oz {

constexpr int kRecElemsPerThread = 4;   // four consecutive i per thread: one 16-byte load per plane

__global__ __launch_bounds__(256) void recompose_kernel(const int32_t* __restrict__ P,
                                                        const int32_t* __restrict__ eA,
                                                        const int32_t* __restrict__ eB, int64_t m,
                                                        int64_t mp, int64_t np, int64_t kp, int s_cap,
                                                        double alpha, double beta,
                                                        double* __restrict__ C, int64_t ldc,
                                                        const Record* rec,
                                                        const int32_t* __restrict__ tile_S, int64_t j_first) {
    if (rec->res.fallback) return;
    const int S_all = rec->res.slices_used;
    const int64_t kblk = ((int64_t(1) << 17) - 1) / S_all / 256 * 256;   // k-blocks of the call's largest count
    const int nkb = int((kp + kblk - 1) / kblk);
    const int64_t j = blockIdx.y;
    const int64_t i0 = (int64_t(blockIdx.x) * 256 + threadIdx.x) * kRecElemsPerThread;
    if (i0 >= m) return;
    // per-tile mode: the block of C this element lies in walked only its own anti-diagonals
    // (four consecutive i never straddle a block: kTile is a multiple of 4)
    const int S = tile_S ? min(tile_S[((j_first + j) / kTile) * (mp / kTile) + i0 / kTile], S_all) : S_all;
    const int eb = eB[j];
    const int64_t plane = np * mp;
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const i32x4* p = reinterpret_cast<const i32x4*>(P + j * mp + i0);   // mp and i0 are multiples of 4
    double R[4] = {0.0, 0.0, 0.0, 0.0};
    for (int kb = 0; kb < nkb; ++kb) {
        double Rb[4] = {0.0, 0.0, 0.0, 0.0};
        for (int d = S - 1; d >= 0; --d) {
            // the planes are read once: streaming loads keep them out of the way of C
            const i32x4 v = __builtin_nontemporal_load(&p[((int64_t(kb) * s_cap + d) * plane) / 4]);
            Rb[0] = double(v.x) + Rb[0] * 0x1p-8;
            Rb[1] = double(v.y) + Rb[1] * 0x1p-8;
            Rb[2] = double(v.z) + Rb[2] * 0x1p-8;
            Rb[3] = double(v.w) + Rb[3] * 0x1p-8;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) R[q] = R[q] + Rb[q];
    }
    const int4 ea4 = *reinterpret_cast<const int4*>(eA + i0);
    const int ea[4] = {ea4.x, ea4.y, ea4.z, ea4.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int64_t i = i0 + q;
        if (i >= m) break;
        const int sc = (ea[q] > kExpAllZero ? ea[q] : 0) + (eb > kExpAllZero ? eb : 0) + (2 * kHeadroomBits - 12);
        const double ab = ldexp(R[q], sc);
        double out = __dmul_rn(alpha, ab);
        if (beta != 0.0) out = __dadd_rn(out, __dmul_rn(beta, C[j * ldc + i]));
        C[j * ldc + i] = out;
    }
}

// C = beta * C (beta == 0 stores zeros without reading C)
__global__ __launch_bounds__(256) void scale_c_kernel(int64_t m, double beta, double* __restrict__ C,
                                                      int64_t ldc) {
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int64_t j = blockIdx.y;
    if (i >= m) return;
    C[j * ldc + i] = (beta == 0.0) ? 0.0 : __dmul_rn(beta, C[j * ldc + i]);
}

void launch_recompose(hipStream_t st, const Workspace& w, const Problem& p, double alpha, double beta,
                      double* C, int64_t ldc) {
    const unsigned gx = unsigned((p.m + 256 * kRecElemsPerThread - 1) / (256 * kRecElemsPerThread));
    for (int64_t j0 = 0; j0 < p.n; j0 += 65535) {
        const unsigned gy = unsigned(p.n - j0 < 65535 ? p.n - j0 : 65535);
        hipLaunchKernelGGL(recompose_kernel, dim3(gx, gy), dim3(256), 0, st, w.P + j0 * p.mp, w.eA, w.eB + j0,
                           p.m, p.mp, p.np, p.kp, p.s_cap, alpha, beta, C + j0 * ldc, ldc, w.rec,
                           p.tile_mode ? w.tile_S : nullptr, j0);
    }
}

void launch_scale_c(hipStream_t st, int64_t m, int64_t n, double beta, double* C, int64_t ldc) {
    const unsigned gx = unsigned((m + 255) / 256);
    for (int64_t j0 = 0; j0 < n; j0 += 65535) {
        const unsigned gy = unsigned(n - j0 < 65535 ? n - j0 : 65535);
        hipLaunchKernelGGL(scale_c_kernel, dim3(gx, gy), dim3(256), 0, st, m, beta, C + j0 * ldc, ldc);
    }
}

}  // namespace oz
