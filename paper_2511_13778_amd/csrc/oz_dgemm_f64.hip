// Native FP64 GEMM on the FP64 matrix instruction: the path the guard falls back to.
// (paper: sections "Pre-processing and Safety Checks" and "Heuristic run time Selection":
//  Inf/NaN in the inputs, an exponent span beyond the available bits, or a slice count outside
//  the efficient range route the call to the native FP64 GEMM.)
//
//   C = alpha * op(A) * op(B) + beta * C,  ordinary floating-point accumulation over k.
//
// v_mfma_f64_16x16x4_f64; 128x128 tile per workgroup, 4 waves of 64x64 (4x4 MFMA tiles),
// K step 16 through double-buffered LDS.  op(B) feeds the row operand and op(A) the column
// operand so that the result's lane index runs along i and stores to column-major C coalesce.
// LDS banks: a tile row (one k) is 130 doubles = 260 dwords, i.e. 4 banks further per k.  The MFMA
// operand reads pair lane groups whose k differ by 8 (= 32 banks): MFMA number kk of a K step
// multiplies k = {kk, kk+8, kk+4, kk+12}, the same set for both operands; they are conflict-free.
// Stores of a k-contiguous operand (16 lanes on 16 different k, same row index) keep a two-way conflict
// on the 32-bank store path (the counters show exactly 4 extra cycles per store); other row lengths
// (129, 131, 133) give the same run time, so it is left as it is.
// Tile loads go through a buffer descriptor (no vector address arithmetic in the K loop); ragged sizes
// run the same loop with clamped rows and a short first K step; products with few tiles, or with a number
// of tiles that is not a whole number of rounds, may split k over several workgroups per tile when the
// caller provides scratch memory (partial tiles added in a fixed order by dgemm_f64_reduce_kernel).
// The kernel is launched on every call and returns at once unless the verdict selected it.
#include "oz_internal.h"

namespace oz {

typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int kDK = 16;
constexpr int kDPad = 2;                        // doubles of padding per LDS row (see the bank note above)
// The tile is T x T with T = 128 (the fast path) or T = 64 (outputs too small to give 128-tiles to
// every CU).  Per thread and operand a K step has T/16 elements; a wave owns (T/2) x (T/2).

// tile loader: 16 (k) x 128 (r) elements of an operand whose element (r, l) is at
// base[r*stride_r + l*stride_l]; out-of-range elements are zero.  8 values per thread.
template <bool ROWS_CONTIG, int T>
__device__ __forceinline__ void dg_load(double (&v)[T / 16], const double* __restrict__ X, int64_t stride_r,
                                        int64_t stride_l, int64_t r0, int64_t rows, int64_t l0, int64_t k) {
#pragma unroll
    for (int q = 0; q < T / 16; ++q) {
        int rr, ll;
        if (ROWS_CONTIG) { rr = threadIdx.x & (T - 1); ll = threadIdx.x / T + (256 / T) * q; }
        else { ll = threadIdx.x & 15; rr = (threadIdx.x >> 4) + 16 * q; }
        const int64_t r = r0 + rr, l = l0 + ll;
        // clamped address + select: the load is unconditional, so the loop stays branch-free
        const int64_t rc = r < rows ? r : rows - 1, lc = l < k ? l : k - 1;
        const double x = X[rc * stride_r + lc * stride_l];
        v[q] = (r < rows && l < k) ? x : 0.0;
    }
}
// interior tiles (no bounds to check): `u` is the wave-uniform address of the K step of this tile,
// `vo` this thread's byte offset inside it (fixed for the whole kernel), the elements of a thread are
// qstep_bytes apart.  The loads go through a buffer descriptor built on `u` (48-bit base in scalar
// registers, element distance as the instruction's scalar offset, `vo` as its 32-bit lane offset), so a
// K step has no vector address arithmetic at all.  Written as plain loads from `u + q*qstep + vo` the
// compiler keeps a 64-bit per-lane address for every element and rebuilds all of them with 64-bit
// vector adds in every K step: some forty vector instructions that compete with the MFMAs for the
// issue slot (measured at 8192^3: 15.36 ms with those, 14.70 ms with the descriptor form).
// The descriptor covers 4 GiB from `u` (raw buffer, no swizzle); the launcher sends operands whose
// offsets could exceed that to the bounds-checked path.
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
// PER_Q: every element of a thread has a lane offset of its own (ragged tiles of a k-contiguous
// operand, whose rows are clamped one by one); otherwise one lane offset and q * qstep_bytes.
template <int T, bool PER_Q>
__device__ __forceinline__ void dg_load_fast(double (&v)[T / 16], const double* u, const uint32_t (&vo)[PER_Q ? T / 16 : 1],
                                             uint32_t qstep_bytes) {
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<double*>(u), 0, -1, 0x00020000);
#pragma unroll
    for (int q = 0; q < T / 16; ++q) {
        const v2u x = __builtin_amdgcn_raw_buffer_load_b64(r, int(vo[PER_Q ? q : 0]),
                                                           PER_Q ? 0 : int(uint32_t(q) * qstep_bytes), 0);
        v[q] = __builtin_bit_cast(double, x);
    }
}
// lane offsets (bytes) of a thread's elements inside a K step of a tile that has `vr` (1..T) valid rows:
// rows past the last valid one are read from the last valid one instead (their products land in rows
// or columns of C that are never stored), so every address stays inside the operand
template <bool ROWS_CONTIG, int T, bool PER_Q>
__device__ __forceinline__ void dg_lane_offsets(uint32_t (&vo)[PER_Q ? T / 16 : 1], int64_t stride_r, int64_t stride_l,
                                                int vr) {
    if (ROWS_CONTIG) {
        const int rr = min(int(threadIdx.x & (T - 1)), vr - 1);
        vo[0] = uint32_t(rr * stride_r + (threadIdx.x / T) * stride_l) * 8u;
    } else {
#pragma unroll
        for (int q = 0; q < (PER_Q ? T / 16 : 1); ++q) {
            const int rr = min(int(threadIdx.x >> 4) + 16 * q, vr - 1);
            vo[q] = uint32_t(rr * stride_r + (threadIdx.x & 15) * stride_l) * 8u;
        }
    }
}

template <bool ROWS_CONTIG, int T>
__device__ __forceinline__ void dg_store(const double (&v)[T / 16], double* lds) {
#pragma unroll
    for (int q = 0; q < T / 16; ++q) {
        int rr, ll;
        if (ROWS_CONTIG) { rr = threadIdx.x & (T - 1); ll = threadIdx.x / T + (256 / T) * q; }
        else { ll = threadIdx.x & 15; rr = (threadIdx.x >> 4) + 16 * q; }
        lds[ll * (T + kDPad) + rr] = v[q];
    }
}

// MODE 0: m, n multiples of the tile and k of the K step.  MODE 1: any m, n, k: edge tiles clamp their
// rows in the (loop-invariant) lane offsets and k % 16 is taken as a short first K step, loaded by the
// bounds-checked loader once per tile; the K loop itself is the same as in MODE 0.  MODE 2: the
// bounds-checked loader with 64-bit indexing everywhere (operands whose leading dimension does not
// fit the 32-bit offsets of the fast loads).
template <bool A_ROWS_CONTIG, bool B_ROWS_CONTIG, int MODE, int T>
__global__ __launch_bounds__(256, 2) void dgemm_f64_kernel(
    const Record* rec, int64_t m, int64_t n, int64_t k, double alpha, const double* __restrict__ A,
    int64_t a_sr, int64_t a_sl, const double* __restrict__ B, int64_t b_sr, int64_t b_sl, double beta,
    double* __restrict__ C, int64_t ldc, int ntm, int ntn, int zsplit, int64_t kpart, double* __restrict__ partial) {
    constexpr bool EDGE = MODE == 2;                       // bounds-checked loads in the K loop
    constexpr bool RAGGED = MODE != 0;                     // bounds-checked stores of C
    constexpr bool A_PER_Q = MODE == 1 && !A_ROWS_CONTIG, B_PER_Q = MODE == 1 && !B_ROWS_CONTIG;
    constexpr int kDLd = T + kDPad;      // LDS row length
    constexpr int WT = T / 2;            // wave tile
    constexpr int MT = WT / 16;          // MFMA tiles per wave and direction
    constexpr int EPT = T / 16;          // elements per thread, operand and K step
    __shared__ double At[2][kDK * kDLd];
    __shared__ double Bt[2][kDK * kDLd];
    if (rec && !rec->res.fallback) return;

    // Workgroup ids are dealt round-robin to the 8 XCDs; each XCD gets a contiguous range of a tile
    // order in which 64 consecutive tiles (what an XCD runs at a time: 32 CUs, two workgroups each)
    // form an 8 x 8 block, so they share 16 panels in that XCD's L2.
    // With a k split (zsplit > 1) a work unit is (tile, part of the k range), ordered part by part.
    int ti, tj, z;
    {
        const int tiles = ntm * ntn, total = tiles * zsplit;
        const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
        const int per = total >> 3, rem = total & 7;
        const int unit = xcd * per + min(xcd, rem) + slot;
        z = unit / tiles;
        const int lin = unit - z * tiles;
        constexpr int GW = 8;
        const int panel = lin / (GW * ntm);
        const int in_panel = lin - panel * GW * ntm;
        const int w = min(GW, ntn - panel * GW);
        ti = in_panel / w;
        tj = panel * GW + in_panel % w;
    }
    const int64_t i0 = int64_t(ti) * T, j0 = int64_t(tj) * T;
    // this unit's k range: part 0 is [0, k - (zsplit-1)*kpart) and carries k mod 16, the others have kpart
    // (a multiple of 16) each; from here on A, B and k describe that range alone
    if (zsplit > 1) {
        const int64_t k0 = k - int64_t(zsplit - 1) * kpart;
        const int64_t kb = z == 0 ? 0 : k0 + int64_t(z - 1) * kpart;
        A += kb * a_sl;
        B += kb * b_sl;
        k = z == 0 ? k0 : kpart;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wi = wave & 1, wj = wave >> 1;

    v4d acc[MT][MT];   // [fj][fi]
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) acc[a][b] = v4d{0.0, 0.0, 0.0, 0.0};

    double va[EPT], vb[EPT];
    const double* ua = A + i0 * a_sr;   // wave-uniform: start of this tile's rows at k = 0
    const double* ub = B + j0 * b_sr;
    uint32_t voa[A_PER_Q ? EPT : 1], vob[B_PER_Q ? EPT : 1];
    dg_lane_offsets<A_ROWS_CONTIG, T, A_PER_Q>(voa, a_sr, a_sl, MODE == 1 ? int(min(int64_t(T), m - i0)) : T);
    dg_lane_offsets<B_ROWS_CONTIG, T, B_PER_Q>(vob, b_sr, b_sl, MODE == 1 ? int(min(int64_t(T), n - j0)) : T);
    const uint32_t qa = uint32_t(A_ROWS_CONTIG ? (256 / T) * a_sl : 16 * a_sr) * 8u;   // bytes between a thread's elements
    const uint32_t qb = uint32_t(B_ROWS_CONTIG ? (256 / T) * b_sl : 16 * b_sr) * 8u;
    // length of the first K step: k % 16 (a full step when that is zero); only MODE 1 has a short one
    const int kfirst = (MODE == 1 && (k & (kDK - 1))) ? int(k & (kDK - 1)) : kDK;
    if (EDGE || kfirst != kDK) {
        dg_load<A_ROWS_CONTIG, T>(va, A, a_sr, a_sl, i0, m, 0, EDGE ? k : kfirst);
        dg_load<B_ROWS_CONTIG, T>(vb, B, b_sr, b_sl, j0, n, 0, EDGE ? k : kfirst);
    } else {
        dg_load_fast<T, A_PER_Q>(va, ua, voa, qa);
        dg_load_fast<T, B_PER_Q>(vb, ub, vob, qb);
    }
    dg_store<A_ROWS_CONTIG, T>(va, At[0]);
    dg_store<B_ROWS_CONTIG, T>(vb, Bt[0]);
    __syncthreads();

    // fragments of MFMA step kk of the K step in LDS buffer `b`: lane group g = lane/16 multiplies
    // k = kk + 8*(g&1) + 4*(g>>1) (see the bank note at the top)
    const int g = lane >> 4;
    const int krow = (8 * (g & 1) + 4 * (g >> 1)) * kDLd;
    const int la_off = wi * WT + (lane & 15) + krow, lb_off = wj * WT + (lane & 15) + krow;
#define OZ_DG_READ(fa, fb, b, kk)                                                              \
    _Pragma("unroll") for (int f = 0; f < MT; ++f) {                                           \
        fa[f] = At[b][la_off + (kk) * kDLd + f * 16];                                          \
        fb[f] = Bt[b][lb_off + (kk) * kDLd + f * 16];                                          \
    }
#define OZ_DG_MFMA(fa, fb)                                                                     \
    _Pragma("unroll") for (int fj = 0; fj < MT; ++fj) _Pragma("unroll") for (int fi = 0; fi < MT; ++fi) \
        acc[fj][fi] = __builtin_amdgcn_mfma_f64_16x16x4f64(fb[fj], fa[fi], acc[fj][fi], 0, 0, 0);

    // Software pipeline of one K step (16 k = 4 MFMA steps of 16 MFMAs), arranged so that the matrix
    // unit always has work.  Interior tiles run it branch-free (the last K step loads its own tile
    // again and stores it where nobody reads it), which leaves one scheduling region per half, and
    // the group barriers below fix the interleave inside it:
    //   step 0: one global load of the next tile per MFMA          (fragments of step 1 are read first)
    //   step 1: MFMAs only                                         (fragments of step 2 are read first)
    //   step 2: one LDS store of the next tile per MFMA            (fragments of step 3 are read first)
    //   barrier: next tile visible, nobody reads this buffer any more (step 3 is in registers)
    //   step 3: MFMAs; they cover the barrier and the first fragment read of the next tile
    double xa[MT], xb[MT], ya[MT], yb[MT];
    int buf = 0;
    OZ_DG_READ(xa, xb, 0, 0);
    // K steps: [0, kfirst), then full steps of 16.  l0 is where the current step ends = the next one starts
    int64_t adv = kfirst;               // distance from the current step's start to the next one's
    for (int64_t l0 = kfirst;; l0 += kDK) {
        const bool have_next = l0 < k;
        if (EDGE) {
            if (have_next) {
                dg_load<A_ROWS_CONTIG, T>(va, A, a_sr, a_sl, i0, m, l0, k);
                dg_load<B_ROWS_CONTIG, T>(vb, B, b_sr, b_sl, j0, n, l0, k);
            }
        } else {
            // the last K step loads its own tile again (valid addresses, stored where nobody reads it)
            ua += have_next ? adv * a_sl : 0;
            ub += have_next ? adv * b_sl : 0;
            adv = kDK;
            dg_load_fast<T, A_PER_Q>(va, ua, voa, qa);
            dg_load_fast<T, B_PER_Q>(vb, ub, vob, qb);
        }
        OZ_DG_READ(ya, yb, buf, 1);
        OZ_DG_MFMA(xa, xb);
        OZ_DG_READ(xa, xb, buf, 2);
        OZ_DG_MFMA(ya, yb);
        OZ_DG_READ(ya, yb, buf, 3);
        if (!EDGE || have_next) {
            dg_store<A_ROWS_CONTIG, T>(va, At[buf ^ 1]);
            dg_store<B_ROWS_CONTIG, T>(vb, Bt[buf ^ 1]);
        }
        OZ_DG_MFMA(xa, xb);
        if (!EDGE && T == 128) {
            // masks: 0x008 MFMA, 0x020 global load, 0x100 LDS read, 0x200 LDS write
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
            }
        }
        __syncthreads();
        buf ^= 1;
        if (!EDGE || have_next) { OZ_DG_READ(xa, xb, buf, 0); }
        OZ_DG_MFMA(ya, yb);
        if (!EDGE && T == 128) {
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
        }
        if (!have_next) break;
    }
#undef OZ_DG_READ
#undef OZ_DG_MFMA

    // result register r of tile (fj, fi): j = fj*16 + 4*r + lane/16, i = fi*16 + lane%16
    if (zsplit > 1) {
        // partial product of this part of the k range: tile (ti, tj) of part z, T x T doubles, i contiguous
        double* dst = partial + ((int64_t(z) * ntn + tj) * ntm + ti) * (T * T);
#pragma unroll
        for (int fj = 0; fj < MT; ++fj)
#pragma unroll
            for (int fi = 0; fi < MT; ++fi)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    dst[(wj * WT + fj * 16 + 4 * r + (lane >> 4)) * T + wi * WT + fi * 16 + (lane & 15)] = acc[fj][fi][r];
        return;
    }
#pragma unroll
    for (int fj = 0; fj < MT; ++fj)
#pragma unroll
        for (int fi = 0; fi < MT; ++fi)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t j = j0 + wj * WT + fj * 16 + 4 * r + (lane >> 4);
                const int64_t i = i0 + wi * WT + fi * 16 + (lane & 15);
                if (!RAGGED || (i < m && j < n)) {
                    double out = __dmul_rn(alpha, acc[fj][fi][r]);
                    if (beta != 0.0) out = __dadd_rn(out, __dmul_rn(beta, C[j * ldc + i]));
                    C[j * ldc + i] = out;
                }
            }
}

// C = alpha * (sum of the parts' partial products, in the order of the parts) + beta * C
template <int T>
__global__ __launch_bounds__(256) void dgemm_f64_reduce_kernel(const Record* rec, int64_t m, int64_t n, double alpha,
                                                               double beta, double* __restrict__ C, int64_t ldc, int ntm,
                                                               int ntn, int zsplit, const double* __restrict__ partial) {
    if (rec && !rec->res.fallback) return;
    const int64_t i = int64_t(blockIdx.x) * 256 + threadIdx.x;
    const int64_t j = blockIdx.y;
    if (i >= m) return;
    const int64_t ti = i / T, tj = j / T;
    const double* src = partial + (tj * ntm + ti) * (T * T) + (j - tj * T) * T + (i - ti * T);
    const int64_t part_stride = int64_t(ntn) * ntm * (T * T);
    double sum = src[0];
    for (int z = 1; z < zsplit; ++z) sum = __dadd_rn(sum, src[z * part_stride]);
    double out = __dmul_rn(alpha, sum);
    if (beta != 0.0) out = __dadd_rn(out, __dmul_rn(beta, C[j * ldc + i]));
    C[j * ldc + i] = out;
}

void launch_dgemm_f64(hipStream_t st, const Record* rec, bool ta, bool tb, int64_t m, int64_t n, int64_t k,
                      double alpha, const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
                      double* C, int64_t ldc, void* scratch, size_t scratch_bytes) {
    // op(A)(i,l): N -> A[i + l*lda] (rows contiguous), T -> A[l + i*lda]
    // op(B)(l,j): N -> B[l + j*ldb] (k contiguous),    T -> B[j + l*ldb] (rows contiguous)
    const int64_t a_sr = ta ? lda : 1, a_sl = ta ? 1 : lda;
    const int64_t b_sr = tb ? 1 : ldb, b_sl = tb ? ldb : 1;
    const bool ac = !ta, bc = tb;
    // 64 x 64 tiles when 128 x 128 tiles would leave more than half of the 2 x 256 workgroup slots empty
    const int64_t tiles128 = ((m + 127) / 128) * ((n + 127) / 128);
    int device = 0, num_cu = 256;
    if (hipGetDevice(&device) == hipSuccess) (void)hipDeviceGetAttribute(&num_cu, hipDeviceAttributeMultiprocessorCount, device);
    // the interior path keeps every offset inside a K step of a tile in 32 bits (a lane's own: at most
    // 15 leading dimensions plus a row of the tile; its elements: up to 7 x 16 leading dimensions
    // further on; in bytes); operands cut out of a very large parent matrix take the bounds-checked
    // path, which indexes in 64 bits
    const int64_t ld_max = lda > ldb ? lda : ldb;
    const bool wide_ld = (128 * ld_max + 256) * 8 >= (int64_t(1) << 32);
    // Few tiles and a long k (a skinny or small output): with scratch memory at hand, the k range is split
    // over zsplit workgroups per 128 x 128 tile so that the two workgroup slots of every CU are filled;
    // the parts leave partial products in the scratch memory and a second kernel adds them in the order
    // of the parts (deterministic) and applies alpha and beta.  Each part gets at least 512 of k.
    int zsplit = 1;
    int64_t kpart = 0;
    if (tiles128 < num_cu && !wide_ld && scratch != nullptr) {
        int64_t z = (2 * int64_t(num_cu)) / tiles128;
        if (z > 16) z = 16;
        if (z > k / 512) z = k / 512;
        const int64_t fit = int64_t(scratch_bytes / (size_t(tiles128) * 128 * 128 * 8));
        if (z > fit) z = fit;
        // A 64 x 64 tile's K step takes about 0.3 of a 128 x 128 tile's, so against the unsplit 64 x 64 path a
        // split pays from four parts on, or from two if the parts give every CU a workgroup (measured:
        // 512 x 512 x 8192 with 5 parts 0.20 ms against 0.40 ms; 1024^3 with 2 parts is slower than unsplit)
        if (z >= 4 || (z >= 2 && z * tiles128 >= num_cu)) {
            zsplit = int(z);
            kpart = k / z / kDK * kDK;
        }
    }
    // Enough tiles for every CU, but not a whole number of rounds (a CU runs two 128 x 128 tiles at a time and
    // a launch lasts as long as the CU with the most tiles): a k split makes the work units smaller, so the
    // last round wastes less.  Estimate per part count z: ceil(tiles * z / CUs) units of 2 * 128 * 128 * k / z
    // flops on a CU that sustains about 289 flops per ns, plus (z + 2) passes over C for the partial tiles at
    // 4.5 TB/s.  Taken when it saves at least 5 % (3072^3: 3 rounds of 576 tiles become 9 / 4 with z = 4).
    if (zsplit == 1 && tiles128 >= num_cu && !wide_ld && scratch != nullptr) {
        auto estimate_ns = [&](int64_t z) -> double {
            const int64_t units_per_cu = (tiles128 * z + num_cu - 1) / num_cu;
            return double(units_per_cu) * (2.0 * 128 * 128 * double(k) / double(z)) / 289.0 +
                   (z > 1 ? double(z + 2) * double(m) * double(n) * 8.0 / 4500.0 : 0.0);
        };
        const int64_t fit = int64_t(scratch_bytes / (size_t(tiles128) * 128 * 128 * 8));
        int64_t best = 1;
        for (int64_t z = 2; z <= 8 && z <= k / 512 && z <= fit; ++z)
            if (estimate_ns(z) < estimate_ns(best)) best = z;
        if (best > 1 && estimate_ns(best) < 0.95 * estimate_ns(1)) {
            zsplit = int(best);
            kpart = k / best / kDK * kDK;
        }
    }
    const bool small = tiles128 < num_cu && zsplit == 1;
    const int T = small ? 64 : 128;
    const int ntm = int((m + T - 1) / T), ntn = int((n + T - 1) / T);
    const dim3 grid(unsigned(ntm) * unsigned(ntn) * unsigned(zsplit)), block(256);
    double* partial = static_cast<double*>(scratch);
    // k < 16: the fast loads always fetch a full K step, which such a matrix does not have
    const int mode = (wide_ld || k < kDK) ? 2 : (((m % T) || (n % T) || (k % kDK)) ? 1 : 0);
#define OZ_DG_M(AC, BC, MODE, TT)                                                                              \
    hipLaunchKernelGGL((dgemm_f64_kernel<AC, BC, MODE, TT>), grid, block, 0, st, rec, m, n, k, alpha, A, a_sr, \
                       a_sl, B, b_sr, b_sl, beta, C, ldc, ntm, ntn, zsplit, kpart, partial)
#define OZ_DG_T(AC, BC, TT)                                                                                    \
    {                                                                                                          \
        if (mode == 2) OZ_DG_M(AC, BC, 2, TT);                                                                 \
        else if (mode == 1) OZ_DG_M(AC, BC, 1, TT);                                                            \
        else OZ_DG_M(AC, BC, 0, TT);                                                                           \
    }
#define OZ_DG(AC, BC)                                                                                          \
    {                                                                                                          \
        if (small) OZ_DG_T(AC, BC, 64) else OZ_DG_T(AC, BC, 128)                                               \
    }
    if (ac && bc) OZ_DG(true, true)
    else if (ac && !bc) OZ_DG(true, false)
    else if (!ac && bc) OZ_DG(false, true)
    else OZ_DG(false, false)
#undef OZ_DG_T
#undef OZ_DG_M
#undef OZ_DG
    if (zsplit > 1) {
        const unsigned gx = unsigned((m + 255) / 256);
        // n < 128 * 256 here (fewer than 256 tiles of 128 columns), so n fits grid.y
        hipLaunchKernelGGL((dgemm_f64_reduce_kernel<128>), dim3(gx, unsigned(n)), dim3(256), 0, st, rec, m, n, alpha, beta,
                           C, ldc, ntm, ntn, zsplit, partial);
    }
}

}  // namespace oz
