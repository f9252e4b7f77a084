// Pre-pass over op(A) and op(B): Inf/NaN scan, per-block exponent Max/Min tables for the
// coarsened ESC, and the row / column exponents the slicing aligns to (integer atomicMax over the
// block maxima: order-free, hence deterministic).
// (paper: sections "Pre-processing and Safety Checks" and "Exponent Span Estimation";
//  block Max/Min: section "ESC", the paragraph on blocks of length b.)
//
// HBM-bound: every FP64 element is read once (8 B), two int16 are written per block of b.
#include "oz_internal.h"

namespace oz {

// exp(x) = floor(log2|x|) from the bit pattern; zero -> is_zero; all-ones field -> bad.
__device__ __forceinline__ int exponent_of(uint64_t bits, bool& is_zero, bool& bad) {
    const uint64_t mag = bits & 0x7FFFFFFFFFFFFFFFull;
    const int field = int(mag >> 52);
    is_zero = (mag == 0);
    bad = (field == 0x7FF);
    if (field != 0) return field - 1023;
    // denormal: value = frac * 2^-1074, exponent = position of the leading one - 1074
    return is_zero ? 0 : (63 - __builtin_clzll(mag)) - 1074;
}

struct BlockStat {
    int mx;        // max exponent over non-zero entries
    int mn;        // min exponent over non-zero entries
    int any_nz;    // block has a non-zero entry
    int any_zero;  // block has a zero entry
    __device__ __forceinline__ void reset() { mx = -32768; mn = 32767; any_nz = 0; any_zero = 0; }
    __device__ __forceinline__ void add(uint64_t bits, int& bad_acc) {
        bool z, bad;
        const int e = exponent_of(bits, z, bad);
        bad_acc |= int(bad);
        if (z) { any_zero = 1; } else { any_nz = 1; mx = max(mx, e); mn = min(mn, e); }
    }
    __device__ __forceinline__ int16_t table_max() const { return int16_t(any_nz ? mx : kExpAllZero); }
    __device__ __forceinline__ int16_t table_min() const {
        return int16_t(!any_nz ? kExpAllZero : (any_zero ? kExpZeroInMin : mn));
    }
};

// resets the control record and the row / column exponents (targets of atomicMax in the scans)
__global__ __launch_bounds__(256) void init_kernel(Record* rec, int32_t* eA, int64_t mp, int32_t* eB, int64_t np,
                                                   int32_t* tile_span, int64_t tiles) {
    const int64_t t = int64_t(blockIdx.x) * 256 + threadIdx.x;
    if (t == 0) {
        rec->infnan = 0;
        rec->span_max = 0;
        rec->esc_exact = 0;
        rec->pair_acc = 0;
        rec->smin_acc = kMaxSlices;
    }
    if (t < tiles) tile_span[t] = 0;
    if (t < 8) {
        rec->tile_sync[t] = 0;
    }
    if (t < mp) eA[t] = kExpAllZero;
    if (t < np) eB[t] = kExpAllZero;
}

// Rows contiguous in memory (stride_r == 1): one thread per row, lanes along the rows, so
// every load instruction of a wave reads 512 contiguous bytes.
// grid: (rows_p/256, ceil(G/kBlocksPerWg)); tab is [2G][rows_p].
constexpr int kScanBlocksPerWg = 4;

__global__ __launch_bounds__(256) void scan_rows_contig_kernel(
    const double* __restrict__ X, int64_t stride_l, int64_t rows, int64_t rows_p, int64_t k,
    int b, int G, int16_t* __restrict__ tab, int max_half, int32_t* __restrict__ e_out, Record* rec,
    int check) {
    const int64_t r = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int g0 = blockIdx.y * kScanBlocksPerWg;
    int bad = 0;
    int row_max = kExpAllZero;
    for (int g = g0; g < min(G, g0 + kScanBlocksPerWg); ++g) {
        BlockStat st;
        st.reset();
        if (r < rows) {
            const int64_t l0 = int64_t(g) * b;
            const int64_t l1 = min(k, l0 + b);
            const uint64_t* src = reinterpret_cast<const uint64_t*>(X) + r + l0 * stride_l;
#pragma unroll 8
            for (int64_t l = l0; l < l1; ++l, src += stride_l) st.add(*src, bad);
        }
        tab[(int64_t(max_half ? g : G + g)) * rows_p + r] = st.table_max();
        tab[(int64_t(max_half ? G + g : g)) * rows_p + r] = st.table_min();
        row_max = max(row_max, int(st.table_max()));
    }
    if (row_max > kExpAllZero) atomicMax(&e_out[r], row_max);
    if (check && bad) atomicOr(&rec->infnan, 1);
}

// k contiguous in memory (stride_l == 1): 16 lanes share one row so that a load instruction
// reads 128 contiguous bytes per row; partial results are combined across the 16 lanes.
// A workgroup covers 16 rows; grid: (rows_p/16, ceil(G/kBlocksPerWg)).
__global__ __launch_bounds__(256) void scan_k_contig_kernel(
    const double* __restrict__ X, int64_t stride_r, int64_t rows, int64_t rows_p, int64_t k,
    int b, int G, int16_t* __restrict__ tab, int max_half, int32_t* __restrict__ e_out, Record* rec,
    int check) {
    int row_max = kExpAllZero;
    const int q = threadIdx.x & 15;
    const int64_t r = int64_t(blockIdx.x) * 16 + (threadIdx.x >> 4);
    const int g0 = blockIdx.y * kScanBlocksPerWg;
    int bad = 0;
    for (int g = g0; g < min(G, g0 + kScanBlocksPerWg); ++g) {
        BlockStat st;
        st.reset();
        if (r < rows) {
            const int64_t l0 = int64_t(g) * b;
            const int64_t l1 = min(k, l0 + b);
            const uint64_t* src = reinterpret_cast<const uint64_t*>(X) + r * stride_r;
#pragma unroll 4
            for (int64_t l = l0 + q; l < l1; l += 16) st.add(src[l], bad);
        }
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) {
            st.mx = max(st.mx, __shfl_xor(st.mx, off));
            st.mn = min(st.mn, __shfl_xor(st.mn, off));
            st.any_nz |= __shfl_xor(st.any_nz, off);
            st.any_zero |= __shfl_xor(st.any_zero, off);
        }
        if (q == 0) {
            tab[(int64_t(max_half ? g : G + g)) * rows_p + r] = st.table_max();
            tab[(int64_t(max_half ? G + g : g)) * rows_p + r] = st.table_min();
            row_max = max(row_max, int(st.table_max()));
        }
    }
    if (q == 0 && row_max > kExpAllZero) atomicMax(&e_out[r], row_max);
    if (check && bad) atomicOr(&rec->infnan, 1);
}

void launch_init(hipStream_t st, const Workspace& w, const Problem& p) {
    const int64_t tiles = (p.mp / kTile) * (p.np / kTile);
    int64_t nmax = p.mp > p.np ? p.mp : p.np;
    if (tiles > nmax) nmax = tiles;
    hipLaunchKernelGGL(init_kernel, dim3(unsigned((nmax + 255) / 256)), dim3(256), 0, st, w.rec, w.eA, p.mp, w.eB, p.np,
                       w.tile_span, tiles);
}

void launch_scan(hipStream_t st, const double* X, int64_t stride_r, int64_t stride_l, int64_t rows,
                 int64_t rows_p, const Problem& p, int16_t* tab, bool max_first, int32_t* e_out,
                 Record* rec, bool check_infnan) {
    const int gy = (p.G + kScanBlocksPerWg - 1) / kScanBlocksPerWg;
    if (stride_r == 1) {
        hipLaunchKernelGGL(scan_rows_contig_kernel, dim3(unsigned(rows_p / 256), gy), dim3(256), 0, st,
                           X, stride_l, rows, rows_p, p.k, p.esc_block, p.G, tab, int(max_first), e_out, rec,
                           int(check_infnan));
    } else {
        hipLaunchKernelGGL(scan_k_contig_kernel, dim3(unsigned(rows_p / 16), gy), dim3(256), 0, st, X,
                           stride_r, rows, rows_p, p.k, p.esc_block, p.G, tab, int(max_first), e_out, rec,
                           int(check_infnan));
    }
}

}  // namespace oz
