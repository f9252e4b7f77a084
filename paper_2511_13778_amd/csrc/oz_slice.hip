// Exponent-aligned slicing of op(A) (per row) and op(B) (per column) into 8-bit two's-complement
// digits with the unsigned-slice encoding.
// (paper: section "ESC" on the per-row shift space; section "Unsigned Slice Encoding": the
//  leading slice is rounded toward -infinity so that the remainder is non-negative, and every
//  sub-leading u8 digit >= 128 is stored as digit-256 with a carry into the next higher digit.)
//
// For an entry a of a row with exponent e_row and S slices:
//   X = floor(a * 2^q),  q = 8S - 3 - e_row,  |X| < 2^(8S-2)   (one headroom bit)
//   X = sum_s d_s 256^(S-1-s),  d_s in [-128, 127].
// a = sgn * M * 2^(E-1075) with the integer significand M, so X = (sgn*M) shifted by
// E - 1075 + q: written here as a 64-bit window W at bit offset o (X = W * 2^o), which covers
// any S up to 26 without multi-word arithmetic.
//
// Output layout (what the INT8 GEMM's tiles load with contiguous 16-byte pieces):
//   slices[s][l/16][r][l%16]  for row r (padded to rows_p), k index l (padded to kp); padding = 0.
// HBM-bound: 8 B read and S bytes written per element.  Operands and slices are touched once per call
// here, so loads and stores carry the streaming (non-temporal) hint: measured 11 % faster.
#include "oz_internal.h"

namespace oz {

struct Fixed {
    int64_t W;
    int o;
};

__device__ __forceinline__ Fixed fixed_point(uint64_t bits, int e_row, int S) {
    const uint64_t mag = bits & 0x7FFFFFFFFFFFFFFFull;
    Fixed f;
    f.W = 0;
    f.o = 0;
    if (mag == 0 || e_row <= kExpAllZero) return f;
    const int field = int(mag >> 52);
    const uint64_t frac = mag & 0x000FFFFFFFFFFFFFull;
    const int64_t M = int64_t(field ? (frac | 0x0010000000000000ull) : frac);
    const int64_t sM = (bits >> 63) ? -M : M;
    const int sh = max(field, 1) - 1075 + (8 * S - 2 - kHeadroomBits - e_row);
    if (sh >= 0) {
        f.W = sM;
        f.o = min(sh, 8 * S);   // only Inf/NaN input (unguarded mode) can reach the clamp
    } else {
        f.W = sM >> min(-sh, 63);   // arithmetic shift: rounds toward -infinity
    }
    return f;
}

// bits [8b, 8b+8) of W * 2^o (two's complement, sign-extended), b = 0 least significant
__device__ __forceinline__ uint32_t byte_of(const Fixed& f, int b) {
    const int p = 8 * b - f.o;
    if (p >= 0) return uint32_t(f.W >> min(p, 63)) & 0xFFu;
    if (p > -8) return (uint32_t(f.W) << (-p)) & 0xFFu;
    return 0u;
}

// Digits of 16 consecutive k of one row, least significant slice first; writes 16 bytes per slice.
__device__ __forceinline__ void emit_slices(const Fixed (&f)[16], int S, int8_t* dst,
                                            int64_t slice_stride) {
    uint32_t carry[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) carry[e] = 0;
    for (int s = S - 1; s >= 0; --s) {
        const int b = S - 1 - s;
        uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const uint32_t u = byte_of(f[e], b) + carry[e];
            carry[e] = (u >= 128u) ? 1u : 0u;       // unused after the leading slice
            w[e >> 2] |= (u & 0xFFu) << (8 * (e & 3));
        }
        *reinterpret_cast<uint4*>(dst + int64_t(s) * slice_stride) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// Up to 8 slices the whole fixed-point value fits one 64-bit word, and the carry chain of the remap
// collapses into one addition: with BIAS = 0x80 in every sub-leading byte, the digits are the bytes
// of X + BIAS with the top bit of every sub-leading byte flipped.
//
// X for S <= 8 without branches: with sh = max(field,1) - 1075 + q (q = 8S - 3 - e_row) it is
// sM << sh or sM >> -sh (arithmetic: rounds toward -infinity), both computed and one selected;
// shift counts are clamped to 63 (a left shift beyond the word only happens for Inf/NaN input in
// unguarded mode).  Zeros, all-zero rows and padding have sM = 0 and need no special case.
__device__ __forceinline__ uint64_t biased_fixed64(uint64_t bits, int q_minus_1075, uint64_t bias) {
    const uint64_t mag = bits & 0x7FFFFFFFFFFFFFFFull;
    const int field = int(mag >> 52);
    const uint64_t frac = mag & 0x000FFFFFFFFFFFFFull;
    const uint64_t M = field ? (frac | 0x0010000000000000ull) : frac;
    const uint64_t sgn = uint64_t(int64_t(bits) >> 63);              // all ones for negative entries
    const int64_t sM = int64_t((M ^ sgn) - sgn);
    const int sh = max(field, 1) + q_minus_1075;
    const int64_t left = sM << min(max(sh, 0), 63);
    const int64_t right = sM >> min(max(-sh, 0), 63);
    return uint64_t(sh >= 0 ? left : right) + bias;
}

// Byte b of 16 values is gathered into four dwords with byte permutes (three per dword).
__device__ __forceinline__ void emit_slices_64(const uint64_t (&bits)[16], int e_row, int S, int8_t* dst,
                                               int64_t slice_stride) {
    const uint64_t bias = S >= 2 ? (0x8080808080808080ull >> (8 * (9 - S))) : 0ull;
    const int q = 8 * S - 2 - kHeadroomBits - (e_row > kExpAllZero ? e_row : 0) - 1075;
    uint32_t lo[16], hi[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const uint64_t y = biased_fixed64(bits[e], q, bias);
        lo[e] = uint32_t(y);
        hi[e] = uint32_t(y >> 32);
    }
    for (int b = S - 1; b >= 0; --b) {
        const uint32_t k = uint32_t(b) & 3u;
        const uint32_t pick = k * 0x0101u + 0x0400u;            // result bytes: [second.k, first.k, -, -]
        const uint32_t flip = (b == S - 1) ? 0u : 0x80808080u;  // the leading digit keeps its sign bit
        uint32_t w[4];
        if (b >= 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t t1 = __builtin_amdgcn_perm(hi[4 * j + 1], hi[4 * j], pick);
                const uint32_t t2 = __builtin_amdgcn_perm(hi[4 * j + 3], hi[4 * j + 2], pick);
                w[j] = __builtin_amdgcn_perm(t2, t1, 0x05040100u) ^ flip;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t t1 = __builtin_amdgcn_perm(lo[4 * j + 1], lo[4 * j], pick);
                const uint32_t t2 = __builtin_amdgcn_perm(lo[4 * j + 3], lo[4 * j + 2], pick);
                w[j] = __builtin_amdgcn_perm(t2, t1, 0x05040100u) ^ flip;
            }
        }
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]},
                                    reinterpret_cast<u32x4*>(dst + int64_t(S - 1 - b) * slice_stride));
    }
}

__device__ __forceinline__ void emit(const uint64_t (&bits)[16], int e_row, int S, int8_t* dst,
                                     int64_t slice_stride) {
    if (S <= 8) {
        emit_slices_64(bits, e_row, S, dst, slice_stride);
    } else {
        Fixed f[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) f[e] = fixed_point(bits[e], e_row, S);
        emit_slices(f, S, dst, slice_stride);
    }
}

constexpr int kSliceChunksPerWg = 1;
constexpr int64_t kMaxGridY = 65535;   // grid.y limit the device reports

// Rows contiguous in memory: thread = row, lanes along rows; loads coalesce across the wave.
// grid: (rows_p/256, chunks of this launch / kSliceChunksPerWg); chunk0 = first 16-k chunk of the launch
__global__ __launch_bounds__(256) void slice_rows_contig_kernel(
    const double* __restrict__ X, int64_t stride_l, int64_t rows, int64_t rows_p, int64_t k,
    int64_t kp, const int32_t* __restrict__ e_row, int8_t* __restrict__ out, const Record* rec,
    int64_t chunk0) {
    if (rec->res.fallback) return;
    const int S = rec->res.slices_used;
    const int64_t r = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int er = e_row[r];
    const int64_t slice_stride = kp * rows_p;      // bytes per slice plane
    // loads are unconditional at clamped addresses (rows >= 1 and k >= 1 here); out-of-range
    // elements are then replaced by zero, so the loop has no divergent branches
    const bool row_ok = r < rows;
    const uint64_t* src = reinterpret_cast<const uint64_t*>(X) + (row_ok ? r : rows - 1);
    for (int cc = 0; cc < kSliceChunksPerWg; ++cc) {
        const int64_t c = chunk0 + int64_t(blockIdx.y) * kSliceChunksPerWg + cc;
        uint64_t bits[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t l = c * 16 + e;
            const uint64_t x = __builtin_nontemporal_load(&src[(l < k ? l : k - 1) * stride_l]);
            bits[e] = (row_ok && l < k) ? x : 0ull;
        }
        emit(bits, er, S, out + (c * rows_p + r) * 16, slice_stride);
    }
}

// k contiguous in memory: a 64-row x 64-k tile is read with lanes along k (512 contiguous bytes
// per wave load), transposed through LDS, then each thread owns (row, 16-k chunk).
// grid: (rows_p/64, kp/64)
__global__ __launch_bounds__(256) void slice_k_contig_kernel(
    const double* __restrict__ X, int64_t stride_r, int64_t rows, int64_t rows_p, int64_t k,
    int64_t kp, const int32_t* __restrict__ e_row, int8_t* __restrict__ out, const Record* rec) {
    __shared__ uint64_t T[64][65];
    if (rec->res.fallback) return;
    const int S = rec->res.slices_used;
    const int64_t r0 = int64_t(blockIdx.x) * 64, l0 = int64_t(blockIdx.y) * 64;
    {
        const int ll = threadIdx.x & 63;
        const int rr0 = threadIdx.x >> 6;
        const uint64_t* src = reinterpret_cast<const uint64_t*>(X);
#pragma unroll
        for (int it = 0; it < 16; ++it) {
            const int rr = rr0 + it * 4;
            const int64_t r = r0 + rr, l = l0 + ll;
            const uint64_t x = __builtin_nontemporal_load(&src[(r < rows ? r : rows - 1) * stride_r + (l < k ? l : k - 1)]);
            T[rr][ll] = (r < rows && l < k) ? x : 0ull;
        }
    }
    __syncthreads();
    const int rr = threadIdx.x & 63, cc = threadIdx.x >> 6;
    const int64_t r = r0 + rr;
    const int er = e_row[r];
    uint64_t bits[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) bits[e] = T[rr][cc * 16 + e];
    const int64_t c = l0 / 16 + cc;
    emit(bits, er, S, out + (c * rows_p + r) * 16, kp * rows_p);
}

void launch_slice(hipStream_t st, const double* X, int64_t stride_r, int64_t stride_l, int64_t rows,
                  int64_t rows_p, const Problem& p, const int32_t* e_row, int8_t* slices,
                  const Record* rec) {
    if (stride_r == 1) {
        // k chunks ride on grid.y: the longest k (2^21) has 131072 of them, launched in slabs
        const int64_t groups = p.kp / 16 / kSliceChunksPerWg;
        for (int64_t g0 = 0; g0 < groups; g0 += kMaxGridY) {
            const unsigned gy = unsigned(groups - g0 < kMaxGridY ? groups - g0 : kMaxGridY);
            hipLaunchKernelGGL(slice_rows_contig_kernel, dim3(unsigned(rows_p / 256), gy), dim3(256), 0, st, X,
                               stride_l, rows, rows_p, p.k, p.kp, e_row, slices, rec, g0 * kSliceChunksPerWg);
        }
    } else {
        hipLaunchKernelGGL(slice_k_contig_kernel, dim3(unsigned(rows_p / 64), unsigned(p.kp / 64)), dim3(256),
                           0, st, X, stride_r, rows, rows_p, p.k, p.kp, e_row, slices, rec);
    }
}

}  // namespace oz
