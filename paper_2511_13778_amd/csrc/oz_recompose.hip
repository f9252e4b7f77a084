// FP64 recomposition of the aggregated anti-diagonal sums and the alpha/beta update.
// (paper: section "FP64 Emulation on Low-Precision Units": slice products are recombined;
//  section "Pre-processing and Safety Checks", second half: partial results are aggregated
//  before the terminal conversion to FP64, so an Inf can only appear in that last step.)
//
// The slice GEMM leaves, per k-block, the exact integer Z = sum_d P_d 256^(S-1-d) as a leading int32
// word T and balanced base-256 digits L_d in [-128,127]:  Z = T 256^(S-1) + sum_{d>=1} L_d 256^(S-1-d).
//
//   AB_ij = 2^(eA_i + eB_j - 10) * sum_kb ( T + sum_{d>=1} 256^-d L_d )
//   C_ij  = alpha * AB_ij + beta * C_ij           (C not read when beta == 0)
//
// Order (fixed, so results are reproducible): k-blocks ascending; inside a k-block from the least
// significant digit, R <- L_d + R * 2^-8, then R <- T + R * 2^-8 (up to seven slices every step but
// this last one is exact: the k-block's value is the exact integer rounded once); block results
// added unscaled; the power of two applied last with ldexp; alpha*AB and beta*C rounded separately,
// then added.
// HBM-bound: (4 + S - 1) * nkb bytes read and 8 (+8 when beta != 0) bytes moved per element of C.
#include "oz_internal.h"

namespace oz {

constexpr int kRecI = 4;   // four consecutive i per thread: one 16-byte load of T per j, of L per digit
constexpr int kRecJ = 4;   // four consecutive j per thread: the four bytes of an L dword

__global__ __launch_bounds__(256) void recompose_kernel(const int32_t* __restrict__ T,
                                                        const int8_t* __restrict__ L,
                                                        const int32_t* __restrict__ eA,
                                                        const int32_t* __restrict__ eB, int64_t m, int64_t n,
                                                        int64_t mp, int64_t np, int64_t kp, int s_cap,
                                                        double alpha, double beta,
                                                        double* __restrict__ C, int64_t ldc,
                                                        const Record* rec,
                                                        const int32_t* __restrict__ tile_S, int64_t j4_first,
                                                        int c_vec) {
    if (rec->res.fallback) return;
    const int S_all = rec->res.slices_used;
    const int64_t kblk = k_block_length(S_all);             // k-blocks of the call's largest count
    const int nkb = int((kp + kblk - 1) / kblk);
    const int64_t j4 = j4_first + blockIdx.y;
    const int64_t j0 = j4 * kRecJ;
    const int64_t i0 = (int64_t(blockIdx.x) * 256 + threadIdx.x) * kRecI;
    if (i0 >= m) return;
    // per-tile mode: the block of C these elements lie in walked only its own anti-diagonals
    // (a 4 x 4 patch never straddles a block: kTile is a multiple of 4)
    const int S = tile_S ? min(tile_S[(j0 / kTile) * (mp / kTile) + i0 / kTile], S_all) : S_all;
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    const i32x4* t4 = reinterpret_cast<const i32x4*>(T);
    const i32x4* l4 = reinterpret_cast<const i32x4*>(L);   // one dword = the four j of one i
    // C is requested first (when it is read at all), then the planes of each k-block in batches: all
    // loads of a batch are in flight together before the first digit is consumed
    double cin[kRecJ][kRecI];
    const bool rows_full = i0 + kRecI <= m;
    // c_vec: C and ldc allow 16-byte accesses (the host checked alignment); used for full groups of four rows
    const bool vec = c_vec && rows_full;
    if (beta != 0.0) {
#pragma unroll
        for (int jj = 0; jj < kRecJ; ++jj) {
            if (vec && j0 + jj < n) {
                const double2* src = reinterpret_cast<const double2*>(C + (j0 + jj) * ldc + i0);
                const double2 lo2 = src[0], hi2 = src[1];
                cin[jj][0] = lo2.x; cin[jj][1] = lo2.y; cin[jj][2] = hi2.x; cin[jj][3] = hi2.y;
            } else {
#pragma unroll
                for (int q = 0; q < kRecI; ++q)
                    cin[jj][q] = (j0 + jj < n && (rows_full || i0 + q < m)) ? C[(j0 + jj) * ldc + i0 + q] : 0.0;
            }
        }
    }
    double R[kRecJ][kRecI];
#pragma unroll
    for (int jj = 0; jj < kRecJ; ++jj)
#pragma unroll
        for (int q = 0; q < kRecI; ++q) R[jj][q] = 0.0;
    constexpr int kBatch = 8;
    for (int kb = 0; kb < nkb; ++kb) {
        // the planes are read once: streaming loads keep them out of the way of C
        i32x4 tv[kRecJ];
#pragma unroll
        for (int jj = 0; jj < kRecJ; ++jj)
            tv[jj] = __builtin_nontemporal_load(&t4[((int64_t(kb) * np + j0 + jj) * mp + i0) / 4]);
        double Rb[kRecJ][kRecI];
#pragma unroll
        for (int jj = 0; jj < kRecJ; ++jj)
#pragma unroll
            for (int q = 0; q < kRecI; ++q) Rb[jj][q] = 0.0;
        for (int d_hi = S - 1; d_hi >= 1; d_hi -= kBatch) {
            i32x4 w[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int d = d_hi - u;
                if (d >= 1)
                    w[u] = __builtin_nontemporal_load(
                        &l4[(((int64_t(kb) * (s_cap - 1) + (d - 1)) * (np / 4) + j4) * mp + i0) / 4]);
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                if (d_hi - u >= 1) {
#pragma unroll
                    for (int q = 0; q < kRecI; ++q)
#pragma unroll
                        for (int jj = 0; jj < kRecJ; ++jj) {
                            const int digit = (w[u][q] << (24 - 8 * jj)) >> 24;       // sign-extended byte jj
                            Rb[jj][q] = double(digit) + Rb[jj][q] * 0x1p-8;
                        }
                }
            }
        }
#pragma unroll
        for (int jj = 0; jj < kRecJ; ++jj)
#pragma unroll
            for (int q = 0; q < kRecI; ++q) R[jj][q] = R[jj][q] + (double(tv[jj][q]) + Rb[jj][q] * 0x1p-8);
    }
    const int4 ea4 = *reinterpret_cast<const int4*>(eA + i0);
    const int ea[4] = {ea4.x, ea4.y, ea4.z, ea4.w};
#pragma unroll
    for (int jj = 0; jj < kRecJ; ++jj) {
        const int64_t j = j0 + jj;
        if (j >= n) break;
        const int eb = eB[j];
        double out[kRecI];
#pragma unroll
        for (int q = 0; q < kRecI; ++q) {
            const int sc = (ea[q] > kExpAllZero ? ea[q] : 0) + (eb > kExpAllZero ? eb : 0) + (2 * kHeadroomBits - 12);
            const double ab = ldexp(R[jj][q], sc);
            out[q] = __dmul_rn(alpha, ab);
            if (beta != 0.0) out[q] = __dadd_rn(out[q], __dmul_rn(beta, cin[jj][q]));
        }
        if (vec) {
            double2* dst = reinterpret_cast<double2*>(C + j * ldc + i0);
            dst[0] = make_double2(out[0], out[1]);
            dst[1] = make_double2(out[2], out[3]);
        } else {
#pragma unroll
            for (int q = 0; q < kRecI; ++q)
                if (i0 + q < m) C[j * ldc + i0 + q] = out[q];
        }
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
    const unsigned gx = unsigned((p.m + 256 * kRecI - 1) / (256 * kRecI));
    const int64_t n4 = (p.n + kRecJ - 1) / kRecJ;
    const int c_vec = (reinterpret_cast<uintptr_t>(C) % 16 == 0 && ldc % 2 == 0) ? 1 : 0;
    for (int64_t j4 = 0; j4 < n4; j4 += 65535) {
        const unsigned gy = unsigned(n4 - j4 < 65535 ? n4 - j4 : 65535);
        hipLaunchKernelGGL(recompose_kernel, dim3(gx, gy), dim3(256), 0, st, w.T, w.L, w.eA, w.eB, p.m, p.n, p.mp,
                           p.np, p.kp, p.s_cap, alpha, beta, C, ldc, w.rec, p.tile_mode ? w.tile_S : nullptr, j4, c_vec);
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
