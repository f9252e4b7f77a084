// Measurement probes (see include/ozprobe.h): the INT8 matrix unit's sustained rate without memory
// traffic, and plain streaming kernels.  They put the roofline fractions of the library's kernels
// next to what this part sustains, and provide dispatches of known size for scaling the memory
// counters.  Built into its own shared library; the product path does not use it.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ozprobe.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// 16 accumulators = the 256 accumulation registers the slice GEMM's waves use; 4 A-fragments and
// 4 B-fragments per lane, as in one K sub-step of that kernel.
__global__ __launch_bounds__(256) void mfma_i8_rate_kernel(int iters, const v4i* __restrict__ data,
                                                           int* __restrict__ out) {
    v4i a[4], b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        a[q] = data[(threadIdx.x * 8 + q) & 4095];
        b[q] = data[(threadIdx.x * 8 + 4 + q + blockIdx.x) & 4095];
    }
    v16i c[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) c[q] = v16i{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int q = 0; q < 16; ++q)
            c[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[q & 3], b[q >> 2], c[q], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += c[q][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
    const size_t stride = size_t(gridDim.x) * 256;
    for (size_t i = size_t(blockIdx.x) * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ src, size_t n, unsigned long long* sink) {
    const size_t stride = size_t(gridDim.x) * 256;
    size_t i = size_t(blockIdx.x) * 256 + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const uint4 p = src[i], q = src[i + stride], r = src[i + 2 * stride], s = src[i + 3 * stride];
        acc ^= p.x ^ p.y ^ p.z ^ p.w ^ q.x ^ q.y ^ q.z ^ q.w ^ r.x ^ r.y ^ r.z ^ r.w ^ s.x ^ s.y ^ s.z ^ s.w;
    }
    for (; i < n; i += stride) {
        const uint4 p = src[i];
        acc ^= p.x ^ p.y ^ p.z ^ p.w;
    }
    if (acc == 0x9E3779B9u) atomicAdd(sink, 1ull);   // data-dependent, practically never taken: keeps the loads alive
}

}  // namespace

extern "C" {

int ozp_launch_mfma_i8(void* stream, const void* operands, void* sink, int iters, int workgroups) {
    if (!operands || !sink || iters < 1 || workgroups < 1 || workgroups > (1 << 20)) return 1;
    hipLaunchKernelGGL(mfma_i8_rate_kernel, dim3(unsigned(workgroups)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       iters, static_cast<const v4i*>(operands), static_cast<int*>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

int ozp_launch_copy(void* stream, void* dst, const void* src, size_t bytes) {
    if (!dst || !src || bytes == 0 || bytes % 16 != 0) return 1;
    hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<uint4*>(dst),
                       static_cast<const uint4*>(src), bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

int ozp_launch_read(void* stream, const void* src, size_t bytes, void* sink) {
    if (!src || !sink || bytes == 0 || bytes % 16 != 0) return 1;
    hipLaunchKernelGGL(read_kernel, dim3(8192), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(src), bytes / 16, static_cast<unsigned long long*>(sink));
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

}  // extern "C"
