/*
 * ozdgemm.h -- C ABI of the MI355X (gfx950) emulated-DGEMM library.
 *
 * C = alpha * op(A) * op(B) + beta * C in FP64, computed with Ozaki scheme I on the INT8
 * matrix units: FP64 operands are aligned per row of op(A) / per column of op(B), cut into
 * 8-bit two's-complement digits ("slices") with the unsigned-slice encoding, the kept slice
 * pairs are multiplied with exact int32 accumulation, and the integer products are recombined
 * in FP64.  A device-resident guard (Inf/NaN scan, Exponent Span Capacity estimate, verdict)
 * chooses the slice count or routes the call to a native FP64 GEMM, with no host-device
 * synchronisation (paper: sections "Unsigned Slice Encoding", "ESC: Exponent Span Capacity
 * Estimation", "ADP: Automatic Dynamic Precision", flowchart of the GEMM decision process).
 *
 * Conventions
 *   - BLAS dgemm semantics, column-major.  op(X) = X for trans 'N'/'n', X^T for 'T'/'t'.
 *     op(A) is m x k, op(B) is k x n, C is m x n.  lda >= max(1, rows of stored A), etc.
 *   - A, B, C, workspace and result are DEVICE pointers owned by the caller.  A and B are only
 *     read.  C is overwritten; it is not read when beta == 0.  The library never allocates or
 *     frees device memory and never synchronises: a call only enqueues kernels on `stream`
 *     (a hipStream_t passed as void*) and returns.
 *   - m == 0 or n == 0: nothing is done.  k == 0 or alpha == 0: C = beta * C.
 *     Limits: m, n <= 2^22, k <= 2^21, m*n*k <= 2^52 (larger sizes are an argument error).
 *   - Return values report host-side argument errors only.  Numerical conditions (Inf/NaN in
 *     the inputs, exponent span too wide, emulation predicted slower) are never errors: they
 *     select the native FP64 path and are recorded in *result.
 *   - Negative zeros in A and B are treated as zero.
 */
#ifndef OZDGEMM_H
#define OZDGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct oz_handle* oz_handle_t;

typedef enum {
    OZ_OK = 0,
    OZ_ERR_ARG = 1,        /* bad trans, negative or too large size, leading dimension too small, bad option */
    OZ_ERR_WORKSPACE = 2,  /* workspace NULL, misaligned (256 B) or smaller than required */
    OZ_ERR_DEVICE = 3,     /* device is not gfx950, or the current device is not the handle's */
    OZ_ERR_HIP = 4         /* a HIP runtime call (launch, event) failed */
} oz_status_t;

/* How the slice count is chosen (section "Performance Evaluation": "no ADP", "ADP forced to
 * 55 bits", "ADP in dynamic mode"; section "Numerical Accuracy": with/without fallback). */
typedef enum {
    OZ_DYNAMIC = 0,         /* scan + ESC; S = ceil((target_bits + ESC + 2) / 8); native FP64 on
                               Inf/NaN, when target_bits + ESC > max_bits, or when the heuristic
                               predicts emulation to be slower */
    OZ_FORCED_GUARDED = 1,  /* scan + ESC run (their cost is paid), S forced from max_bits; only
                               Inf/NaN selects the native path */
    OZ_FIXED_GUARDED = 2,   /* S from max_bits; native path on Inf/NaN, on target_bits + ESC > max_bits, or
                               when the S slices cannot carry target_bits + ESC (S slices carry 8S - 2
                               magnitude bits: ceil((target_bits + ESC + 2) / 8) > S) */
    OZ_FIXED_UNGUARDED = 3, /* S from max_bits; no Inf/NaN test, no ESC, never falls back */
    OZ_NATIVE = 4           /* always the FP64-MFMA GEMM */
} oz_mode_t;

typedef struct {
    int32_t mode;         /* oz_mode_t */
    int32_t target_bits;  /* mantissa bits to preserve for the dominant products (default 53) */
    int32_t max_bits;     /* fixed modes: bits that set S = ceil((max_bits+1)/8) (55 -> 7 slices);
                             guarded/dynamic modes: cap on target_bits + ESC.  1..200 */
    int32_t slices;       /* > 0 overrides the slice count of the fixed/forced modes (1..26) */
    int32_t esc_block;    /* block length b of the coarsened ESC; 0 = 64.  Multiple of 16, <= 1024 */
    int32_t heuristic;    /* OZ_DYNAMIC only: 1 = apply the run-time cost model, 0 = do not.  The model is
                             first evaluated on the host for the smallest slice count any input can
                             get (ESC = 1); if that already loses against FP64 the call runs the
                             native GEMM without scanning A and B: reason 3, esc -1, infnan 0 */
    int32_t tile_slices;  /* OZ_DYNAMIC only: 1 = every 256 x 256 block of C takes the slice count of its
                             own ESC, S_T = ceil((target_bits + ESC_T + 2) / 8): the ESC is a property of
                             a dot product (section "ESC"), and a tighter estimate is what section
                             "Limitations and Future Directions" asks for.  Operands are still sliced
                             once, into max S_T planes; a block multiplies the pairs s + t <= S_T - 1.
                             Fallback decisions stay global (largest ESC); the cost model is fed the
                             mean pair count per block, rounded up.  0 = one slice count for all of C */
} oz_opts_t;

/* Decision record, written to DEVICE memory by the verdict kernel. */
typedef struct {
    int32_t fallback;       /* 0 = emulated, 1 = native FP64 */
    int32_t reason;         /* 0 none, 1 Inf/NaN in A or B, 2 bits > max_bits, 3 heuristic, 4 OZ_NATIVE */
    int32_t slices_used;    /* S of the emulated path, 0 when fallback */
    int32_t esc;            /* coarsened ESC (clamped to 4096), -1 when not computed */
    int32_t required_bits;  /* target_bits + ESC, 0 when not computed */
    int32_t infnan;         /* 1 when the scan saw an all-ones exponent field */
    int32_t slices_min;     /* smallest slice count of any 256 x 256 block of C (== slices_used unless
                               tile_slices); 0 when fallback */
    int32_t reserved_;      /* 0 */
    int64_t pair_tiles;     /* slice-pair products of 256 x 256 blocks of C that the call multiplies:
                               sum over blocks of S_T (S_T + 1) / 2; 0 when fallback */
} oz_result_t;

/* Cost model of the run-time heuristic (section "Heuristic run time Selection"); integer
 * arithmetic so that host, device and any checker agree bit for bit:
 *   t_emu = fixed_ns + (2mnk / int8_ops_per_ns) * S(S+1)/2
 *           + ((16+S)(mk+kn) + (2S+22)mn) / bytes_per_ns,     t_f64 = 2mnk / fp64_flops_per_ns,
 * emulation is "slower" when t_emu > t_f64.  With tile_slices the factor S(S+1)/2 is replaced by the
 * mean pair count per 256 x 256 block of C, rounded up; S in the streaming term is the largest S_T. */
typedef struct {
    int64_t int8_ops_per_ns;
    int64_t fp64_flops_per_ns;
    int64_t bytes_per_ns;
    int64_t fixed_ns;
} oz_heuristic_t;

/* Section "GPU-Resident Integration": the whole decision process lives on the device, so the
 * host-side state is small.  Creates a handle bound to HIP device `device` (must be gfx950): the
 * device's compute-unit count, the cost-model constants of the run-time heuristic, the event
 * pool of the stage timer, the side streams (default priority) and events of the batched call, and
 * the device address of the static workspace of oz_dgemm_static on that device.  Allocates host
 * memory, streams and events, no device memory; *handle is NULL on failure.
 * Errors: OZ_ERR_ARG (handle NULL), OZ_ERR_DEVICE (no such device / not gfx950), OZ_ERR_HIP (the
 * static workspace's address could not be resolved). */
oz_status_t oz_create(oz_handle_t* handle, int device);

/* Releases what oz_create made (host memory, streams, events).  Work already enqueued with the handle is
 * not waited for: it only references caller-owned device memory.  OZ_ERR_ARG on NULL. */
oz_status_t oz_destroy(oz_handle_t handle);

/* Fills *opts with the defaults: OZ_DYNAMIC, target 53, max 200, slices 0, esc_block 0, heuristic 1,
 * tile_slices 1. */
void oz_default_opts(oz_opts_t* opts);

/* Replaces the heuristic's constants (defaults are calibrated for MI355X). */
oz_status_t oz_set_heuristic(oz_handle_t handle, const oz_heuristic_t* model);

/* Sections "Unsigned Slice Encoding" and "ADP" fix what a call stores between its steps: the
 * row/column exponents, the per-block Max/Min exponent tables of the coarsened ESC, the S slice
 * planes of each operand and the S anti-diagonal sums per k-block.  Returns the bytes of device
 * workspace oz_dgemm needs for this problem and these options, sized for the largest slice count
 * the options allow (fixed modes: the S of max_bits/slices; OZ_DYNAMIC: the S of max_bits, or the
 * largest S the cost model still calls faster when heuristic = 1).  Host-only, no device access.
 * Returns 0 on invalid arguments. */
size_t oz_dgemm_workspace_bytes(oz_handle_t handle, char transa, char transb,
                                int64_t m, int64_t n, int64_t k, const oz_opts_t* opts);

/* The emulated DGEMM with guardrails: the flowchart of the GEMM decision process, steps in the
 * order of sections "Pre-processing and Safety Checks" (Inf/NaN scan), "Exponent Span
 * Estimation" (block Max/Min tables, coarsened ESC), "Heuristic run time Selection" (verdict),
 * "Unsigned Slice Encoding" (slicing), "FP64 Emulation on Low-Precision Units" (slice-pair INT8
 * GEMMs, FP64 recomposition), with the native FP64 GEMM as the other branch.  All kernels are
 * enqueued on `stream`; the ones after the verdict read the device-resident record.
 *   A, B, C: device, column-major, leading dimensions in elements (see Conventions above).
 *   workspace: device, 256-byte aligned, >= oz_dgemm_workspace_bytes(...); contents are scratch
 *     on entry and hold the intermediates afterwards (oz_dgemm_layout).  Calls sharing a
 *     workspace must be ordered on one stream.
 *   result: device oz_result_t written by the verdict kernel, may be NULL.
 * Errors (nothing is enqueued): OZ_ERR_ARG, OZ_ERR_WORKSPACE, OZ_ERR_DEVICE; OZ_ERR_HIP if a
 * launch failed. */
oz_status_t oz_dgemm(oz_handle_t handle, void* stream, char transa, char transb,
                     int64_t m, int64_t n, int64_t k, double alpha,
                     const double* A, int64_t lda, const double* B, int64_t ldb,
                     double beta, double* C, int64_t ldc,
                     const oz_opts_t* opts, void* workspace, size_t workspace_bytes,
                     oz_result_t* result);

/* oz_dgemm for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a
 * static device array inside the library, OZ_STATIC_SCRATCH_BYTES per GPU (each GPU the library
 * runs on holds its own copy until the process ends; its address is resolved once per handle in
 * oz_create).  The call allocates nothing and frees nothing: it only enqueues the same kernels as
 * oz_dgemm on `stream`.  All other arguments, conventions and the record are those of oz_dgemm.
 *   - A problem whose oz_dgemm_workspace_bytes(...) exceeds OZ_STATIC_SCRATCH_BYTES is refused
 *     with OZ_ERR_WORKSPACE before anything is enqueued (256 MiB holds e.g. 2048^3 with 7 slices,
 *     or 1024^3 in OZ_DYNAMIC with max_bits = 200).
 *   - The array keeps the previous call's contents; every stage rewrites what it reads, nothing
 *     is assumed to start at zero.
 *   - All calls on one GPU, from any handle or thread, share the one array: calls that overlap in
 *     time on a GPU race.  Order them on one stream (or with events). */
#define OZ_STATIC_SCRATCH_BYTES (256u << 20)
oz_status_t oz_dgemm_static(oz_handle_t handle, void* stream, char transa, char transb,
                            int64_t m, int64_t n, int64_t k, double alpha,
                            const double* A, int64_t lda, const double* B, int64_t ldb,
                            double beta, double* C, int64_t ldc,
                            const oz_opts_t* opts, oz_result_t* result);

/* batch_count independent problems of one shape: problem b uses A + b*stride_a, B + b*stride_b,
 * C + b*stride_c (strides in elements; 0 repeats an operand; the C blocks must not overlap) and
 * writes its own record to results[b] (device array of batch_count records, may be NULL).  Every
 * problem goes through the whole decision process on its own, so slice counts and fallbacks may
 * differ inside a batch (the paper's application runs show a distribution of slice counts over
 * the GEMMs of one factorisation: section "Application-Level Integration").
 * Concurrency follows the workspace: with room for q >= 2 times oz_dgemm_workspace_bytes(...)
 * (each rounded up to 256 bytes) the problems run q at a time, q <= OZ_BATCH_LANES, on streams the
 * handle owns, forked from and joined to `stream` with events (so the call still only enqueues,
 * and everything it enqueued is ordered before later work on `stream`); with room for one they
 * run one after the other on `stream`.  Stage timing (oz_profile_*) records serial batches only.
 * Two batched calls on one handle must not overlap in time (they share the handle's streams).
 * batch_count == 0 is a no-op; errors are those of oz_dgemm, checked before anything is enqueued. */
#define OZ_BATCH_LANES 4
oz_status_t oz_dgemm_strided_batched(oz_handle_t handle, void* stream, char transa, char transb,
                                     int64_t m, int64_t n, int64_t k, double alpha,
                                     const double* A, int64_t lda, int64_t stride_a,
                                     const double* B, int64_t ldb, int64_t stride_b,
                                     double beta, double* C, int64_t ldc, int64_t stride_c,
                                     int64_t batch_count, const oz_opts_t* opts,
                                     void* workspace, size_t workspace_bytes, oz_result_t* results);

/* Complex product by the 4M method (section "Conclusion": the emulated DGEMM and its guardrails
 * extend to ZGEMM via 4M): C = alpha * op(A) * op(B) + beta * C with complex matrices stored
 * interleaved (re, im), column-major, leading dimensions in complex elements; op is 'N', 'T' or
 * 'C' (conjugate transpose).  A and B are split into real and imaginary parts, the four real
 * products  Pr = Ar Br - Ai Bi,  Pi = Ar Bi + Ai Br  run through the emulated DGEMM one after the
 * other on `stream` (each with its own scan, ESC and verdict; the second of each pair accumulates
 * onto the first), and C = alpha (Pr + i Pi) + beta C is formed with every real product and sum
 * rounded separately.  alpha, beta: host pointers to (re, im).  C is not read when beta == 0.
 * results: device array of four records (Ar Br, Ai Bi, Ar Bi, Ai Br) or NULL.  workspace as for
 * oz_dgemm, at least oz_zgemm_workspace_bytes(...) (planar copies of A and B, the planar product,
 * one real call's workspace).  k == 0 gives C = beta C.  Errors as oz_dgemm. */
size_t oz_zgemm_workspace_bytes(oz_handle_t handle, char transa, char transb,
                                int64_t m, int64_t n, int64_t k, const oz_opts_t* opts);
oz_status_t oz_zgemm(oz_handle_t handle, void* stream, char transa, char transb,
                     int64_t m, int64_t n, int64_t k, const double* alpha,
                     const void* A, int64_t lda, const void* B, int64_t ldb,
                     const double* beta, void* C, int64_t ldc,
                     const oz_opts_t* opts, void* workspace, size_t workspace_bytes,
                     oz_result_t* results);

/* Layout of the intermediate buffers inside the workspace after an oz_dgemm call, for
 * inspection by tests (all offsets in bytes from `workspace`):
 *   eA   int32[mp]              row exponents of op(A); -12288 marks an all-zero row
 *   eB   int32[np]              column exponents of op(B)
 *   As   int8 [S_cap][kp/16][mp][16]   slice s of op(A): element (i,l) at
 *                               ((s*(kp/16) + l/16)*mp + i)*16 + l%16; padding is zero
 *   Bs   int8 [S_cap][kp/16][np][16]   slice t of op(B): element (l,j) likewise with j for i
 *   T    int32[nkb][np][mp]     leading word of the aggregated anti-diagonal sums of k-block kb: with
 *                               P_d = sum_{s+t=d} As_s Bs_t^T the exact integer Z = sum_d P_d 256^(S-1-d)
 *                               is T * 256^(S-1) + sum_{d>=1} L_d 256^(S-1-d); element (i,j) at
 *                               (kb*np + j)*mp + i
 *   L    int8 [nkb][S_cap-1][np/4][mp][4]   balanced digit L_d in [-128,127], d >= 1, of element (i,j) at
 *                               (((kb*(S_cap-1) + d-1)*(np/4) + j/4)*mp + i)*4 + j%4
 *   tileS int32[np/256][mp/256]  slice count of block (ti, tj) of C at tj*(mp/256) + ti (written only
 *                               with tile_slices in OZ_DYNAMIC mode); the same number of int32 follows it: the
 *                               order in which the slice GEMM dealt the blocks to its workgroups
 * mp, np = m, n rounded up to 256; kp = k rounded up to 128; kblk = k-block length for S_cap. */
typedef struct {
    int64_t mp, np, kp, s_cap, nkb, kblk;
    size_t off_eA, off_eB, off_As, off_Bs, off_T, off_L, off_record, off_tileS;
    size_t total_bytes;
} oz_layout_t;

oz_status_t oz_dgemm_layout(oz_handle_t handle, char transa, char transb,
                            int64_t m, int64_t n, int64_t k, const oz_opts_t* opts,
                            oz_layout_t* layout);

/* Stage timing with HIP events on the call's own stream.  oz_profile_enable(h, n) makes the
 * next n oz_dgemm calls record an event after every stage; oz_profile_read(h, call, ms)
 * (after the stream has been synchronised by the caller) writes OZ_NUM_STAGES durations in
 * milliseconds.  Stages: 0 scan (Inf/NaN + exponent min/max), 1 ESC, 2 verdict,
 * 3 slicing, 4 slice-pair INT8 GEMMs, 5 FP64 recomposition, 6 native FP64 GEMM. */
#define OZ_NUM_STAGES 7
oz_status_t oz_profile_enable(oz_handle_t handle, int32_t max_calls);
oz_status_t oz_profile_read(oz_handle_t handle, int32_t call, float* stage_ms);

/* The fallback branch of the decision process on its own (sections "Pre-processing and Safety
 * Checks" and "Heuristic run time Selection": the native FP64 GEMM that Inf/NaN inputs, too wide
 * an exponent span or an inefficient slice count route to), and the baseline the paper's speed-ups
 * are quoted against.  Same conventions as oz_dgemm; no workspace, no record; only enqueues.
 * Errors: OZ_ERR_ARG, OZ_ERR_DEVICE, OZ_ERR_HIP. */
oz_status_t oz_native_dgemm(oz_handle_t handle, void* stream, char transa, char transb,
                            int64_t m, int64_t n, int64_t k, double alpha,
                            const double* A, int64_t lda, const double* B, int64_t ldb,
                            double beta, double* C, int64_t ldc);

const char* oz_status_string(oz_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* OZDGEMM_H */
