// Helpers of the complex product by the 4M method (paper: section "Conclusion": the emulated DGEMM
// with its guardrails extends to ZGEMM via 4M): a complex matrix is split into its real and
// imaginary parts, four real products run through the emulated DGEMM, and the parts are combined
// with alpha and beta.  Both kernels are elementwise and HBM-bound.
#include "oz_internal.h"

namespace oz {

// Z (column-major rows x cols of interleaved (re, im), leading dimension ld) ->
// re, im (column-major rows x cols, leading dimension rows); im_sign = -1 takes the conjugate.
__global__ __launch_bounds__(256) void zsplit_kernel(const double2* __restrict__ Z, int64_t ld, int64_t rows,
                                                     double* __restrict__ re, double* __restrict__ im,
                                                     double im_sign) {
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int64_t j = blockIdx.y;
    if (i >= rows) return;
    const double2 z = Z[j * ld + i];
    re[j * rows + i] = z.x;
    im[j * rows + i] = im_sign < 0 ? -z.y : z.y;
}

// C = alpha * (Pr + i Pi) + beta * C on interleaved C; every real product and sum rounded separately,
// in this order:  re = (ar*Pr - ai*Pi) + (br*Cr - bi*Ci),  im = (ar*Pi + ai*Pr) + (br*Ci + bi*Cr).
// C is not read when beta == 0.
__global__ __launch_bounds__(256) void zcombine_kernel(const double* __restrict__ Pr, const double* __restrict__ Pi,
                                                       int64_t m, double ar, double ai, double br, double bi,
                                                       double2* __restrict__ C, int64_t ldc) {
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int64_t j = blockIdx.y;
    if (i >= m) return;
    const double pr = Pr[j * m + i], pi = Pi[j * m + i];
    double re = __dsub_rn(__dmul_rn(ar, pr), __dmul_rn(ai, pi));
    double im = __dadd_rn(__dmul_rn(ar, pi), __dmul_rn(ai, pr));
    if (br != 0.0 || bi != 0.0) {
        const double2 c = C[j * ldc + i];
        re = __dadd_rn(re, __dsub_rn(__dmul_rn(br, c.x), __dmul_rn(bi, c.y)));
        im = __dadd_rn(im, __dadd_rn(__dmul_rn(br, c.y), __dmul_rn(bi, c.x)));
    }
    C[j * ldc + i] = make_double2(re, im);
}

void launch_zsplit(hipStream_t st, const void* Z, int64_t ld, int64_t rows, int64_t cols, double* re, double* im,
                   bool conj) {
    if (rows == 0 || cols == 0) return;
    const unsigned gx = unsigned((rows + 255) / 256);
    for (int64_t j0 = 0; j0 < cols; j0 += 65535) {
        const unsigned gy = unsigned(cols - j0 < 65535 ? cols - j0 : 65535);
        hipLaunchKernelGGL(zsplit_kernel, dim3(gx, gy), dim3(256), 0, st, static_cast<const double2*>(Z) + j0 * ld, ld,
                           rows, re + j0 * rows, im + j0 * rows, conj ? -1.0 : 1.0);
    }
}

void launch_zcombine(hipStream_t st, const double* Pr, const double* Pi, int64_t m, int64_t n, double ar, double ai,
                     double br, double bi, void* C, int64_t ldc) {
    const unsigned gx = unsigned((m + 255) / 256);
    for (int64_t j0 = 0; j0 < n; j0 += 65535) {
        const unsigned gy = unsigned(n - j0 < 65535 ? n - j0 : 65535);
        hipLaunchKernelGGL(zcombine_kernel, dim3(gx, gy), dim3(256), 0, st, Pr + j0 * m, Pi + j0 * m, m, ar, ai, br, bi,
                           static_cast<double2*>(C) + j0 * ldc, ldc);
    }
}

}  // namespace oz
