// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ozdgemm.h"

namespace oz {

// ---- constants of the method -----------------------------------------------------------
constexpr int kHeadroomBits = 1;      // spare bit in the leading digit: |X| < 2^(8S-2)
constexpr int kMaxSlices = 26;        // 200 mantissa bits
constexpr int kEscCap = 4096;         // reported ESC is clamped to this
constexpr int kDefaultEscBlock = 64;
constexpr int64_t kMaxRows = int64_t(1) << 22;   // largest m, n
constexpr int64_t kMaxK = int64_t(1) << 21;      // largest k
constexpr int64_t kMaxMnk = int64_t(1) << 52;    // largest m*n*k: the cost model multiplies 2mnk by up to 351 pairs in int64

// Exponents are kept as int16 in the block tables.  Real exponents lie in [-1074, 1023].
// kExpZeroInMin: Min of a block that holds a zero (exp(0) = -infinity).
// kExpAllZero  : Max and Min of a block without any non-zero entry.
// Sums of two table entries classify a candidate: >= -4096 a real exponent sum,
// [-10000, -4096) "no information", < -10000 "this block contributes nothing to the product".
constexpr int kExpZeroInMin = -6144;
constexpr int kExpAllZero = -12288;
constexpr int kSumRealFloor = -4096;
constexpr int kSumDeadBelow = -10000;

// ---- tiling constants shared between kernels and the workspace layout --------------------
constexpr int kRowPad = 256;          // rows of the slice panels are padded to this
constexpr int kKPad = 128;            // k is padded to this (K tile of the INT8 GEMM)
constexpr int kTile = 256;            // edge of the blocks of C that can take their own slice count
                                      // (= the slice GEMM's workgroup tile; kRowPad is a multiple)

// ---- device-resident control record ---------------------------------------------------
struct Record {
    int32_t infnan;        // set by the scan kernels (atomicOr)
    int32_t span_max;      // max_ij (eA_i + eB_j - zt_ij), set by the ESC kernels (atomicMax)
    int32_t esc_exact;     // set by the MFMA ESC kernel when a pair needs the exact int16 kernel
    int32_t pad_;
    int32_t tile_sync[8];  // per-XCD arrival counters of the slice GEMM's workgroups
    unsigned long long pair_acc;   // per-tile mode: sum over tiles of S_T(S_T+1)/2 (atomicAdd)
    int32_t smin_acc;      // per-tile mode: smallest S_T (atomicMin)
    int32_t pad2_;
    oz_result_t res;       // written by the verdict kernel, read by every later kernel
};

struct Problem {
    int64_t m, n, k;
    int64_t mp, np, kp;    // padded sizes
    int32_t s_cap;         // slice planes the workspace holds
    int32_t nkb;           // number of k-blocks (int32 accumulator headroom)
    int64_t kblk;          // k-block length (multiple of kKPad)
    int32_t esc_block;     // b
    int32_t G;             // ceil(k / b)
    int32_t num_cu;        // compute units of the device
    int32_t tile_mode;     // 1: every kTile x kTile block of C takes its own slice count (OZ_DYNAMIC + tile_slices)
    int32_t raw_slots;     // tiles the raw buffer holds (a launch splits the k range of fewer tiles than there are CUs)
};

struct Workspace {
    Record* rec;
    int32_t* eA;           // [mp]
    int32_t* eB;           // [np]
    int16_t* U;            // [2G][mp]  h <  G: Max exponent of block h of row i of op(A)
                           //           h >= G: Min exponent of block h-G
    int16_t* V;            // [2G][np]  h <  G: Min exponent of block h of column j of op(B)
                           //           h >= G: Max exponent of block h-G
    uint16_t* EU;          // [ceil(2G/32)*4][mp][8] BF16 encoding of U relative to eA
    uint16_t* EV;          // [ceil(2G/32)*4][np][8] BF16 encoding of V relative to eB
    int8_t* As;            // [s_cap][kp/16][mp][16]
    int8_t* Bs;            // [s_cap][kp/16][np][16]
    // aggregated anti-diagonal sums of a k-block: Z = sum_d P_d 256^(S-1-d) = T * 256^(S-1) + sum_{d>=1} L_d 256^(S-1-d)
    int32_t* T;            // [nkb][np][mp]                   leading word (anti-diagonal 0 plus the carry from below)
    int8_t* L;             // [nkb][s_cap-1][np/4][mp][4]     balanced digit of anti-diagonal d >= 1 at plane d-1; four
                           //                                 consecutive j of one i share a dword
    int32_t* raw;          // [nkb][s_cap][raw_slots][kTile][kTile]  unaggregated sums of the tiles whose k range is split
                           //                                 over several workgroups (integer atomics), tile-local [j][i]
    int32_t* tile_span;    // [np/kTile][mp/kTile] largest coarsened span of the block's dot products (atomicMax)
    int32_t* tile_S;       // [np/kTile][mp/kTile] slice count of the block (per-tile mode), followed by as many
                           // entries again: the order in which the slice GEMM deals the tiles to its workgroups
};

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// k-range one int32 accumulator can take: |digit product| <= 2^14, an anti-diagonal sums at most
// S*kblk of them, and the aggregation adds a carry below 2^23 from the less significant
// anti-diagonals: S*kblk*2^14 + 2^23 <= 2^31 - 1.  Multiple of 256.
__host__ __device__ inline int64_t k_block_length(int S) {
    return ((int64_t(1) << 17) - (int64_t(1) << 9) - 1) / S / 256 * 256;
}

// ---- stage launchers (each only enqueues) --------------------------------------------
// element (r, l) of a k-by-rows operand is at base[r*stride_r + l*stride_l]
void launch_init(hipStream_t st, const Workspace& w, const Problem& p);
void launch_scan(hipStream_t st, const double* X, int64_t stride_r, int64_t stride_l,
                 int64_t rows, int64_t rows_p, const Problem& p, int16_t* tab, bool max_first,
                 int32_t* e_out, Record* rec, bool check_infnan);
void launch_esc(hipStream_t st, const Workspace& w, const Problem& p);
// per-tile mode: slice count of every block of C from its span, and the sums the verdict needs
void launch_tile_verdict(hipStream_t st, const Workspace& w, const Problem& p, const oz_opts_t& o);
// kind: 0 unguarded, 1 guarded, 2 nothing to multiply (record says "emulated, 0 slices"),
// 3 native by the cost model alone (nothing scanned)
void launch_verdict(hipStream_t st, const Workspace& w, const Problem& p, const oz_opts_t& o,
                    const oz_heuristic_t& hm, int kind, oz_result_t* user_result);
void launch_slice(hipStream_t st, const double* X, int64_t stride_r, int64_t stride_l,
                  int64_t rows, int64_t rows_p, const Problem& p, const int32_t* e_row,
                  int8_t* slices, const Record* rec);
void launch_gemm_i8(hipStream_t st, const Workspace& w, const Problem& p);
void launch_recompose(hipStream_t st, const Workspace& w, const Problem& p, double alpha,
                      double beta, double* C, int64_t ldc);
// rec == nullptr: run unconditionally; otherwise run only when rec->res.fallback != 0.
// scratch (may be nullptr): device memory the kernel may use for partial products when it splits the
// k range of a product with few tiles; nothing else may use it while the GEMM runs
void launch_dgemm_f64(hipStream_t st, const Record* rec, bool ta, bool tb, int64_t m, int64_t n,
                      int64_t k, double alpha, const double* A, int64_t lda, const double* B,
                      int64_t ldb, double beta, double* C, int64_t ldc, void* scratch = nullptr,
                      size_t scratch_bytes = 0);
void launch_scale_c(hipStream_t st, int64_t m, int64_t n, double beta, double* C, int64_t ldc);
// complex product by the 4M method: split an interleaved complex matrix into planar parts (conj negates
// the imaginary part), and combine the planar product with alpha, beta and the interleaved C
void launch_zsplit(hipStream_t st, const void* Z, int64_t ld, int64_t rows, int64_t cols, double* re, double* im,
                   bool conj);
void launch_zcombine(hipStream_t st, const double* Pr, const double* Pi, int64_t m, int64_t n, double ar, double ai,
                     double br, double bi, void* C, int64_t ldc);

}  // namespace oz
