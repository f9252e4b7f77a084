/*
 * ozprobe.h -- C ABI of the measurement probes that put the library's roofline figures in context
 * (liboz_probe.so; not part of the product path, nothing in liboz_mi355x.so depends on it).
 *
 * The paper reports the slice GEMMs as the dominant cost (section "Performance Evaluation",
 * breakdown of the run time) and gives rates relative to the native FP64 GEMM; to judge a kernel on
 * this part one needs the part's own ceilings under sustained load, which differ from the data-sheet
 * peaks: the matrix unit's rate with operands that toggle like slice digits do, and the memory
 * system's rate for a plain streaming kernel.  Each probe only enqueues one kernel on `stream`;
 * the caller times it (HIP events) and owns all buffers (DEVICE pointers).  Return: 0 ok, 1 bad
 * argument, 4 launch failed.
 */
#ifndef OZPROBE_H
#define OZPROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* INT8 matrix-unit loop with no memory traffic: every wave of `workgroups` x 4 waves issues
 * iters x 16 v_mfma_i32_32x32x32_i8 on 16 independent accumulators; the eight 16-byte operand
 * fragments of a lane are read once from `operands` (>= 65536 bytes: fill with a constant for the
 * "quiet" ceiling or with random bytes for the ceiling under slice-like data).  `sink` receives
 * workgroups*256 int32.  Work: workgroups * 4 * iters * 16 * 65536 int8 ops (multiply-add = 2). */
int ozp_launch_mfma_i8(void* stream, const void* operands, void* sink, int iters, int workgroups);

/* Plain streaming kernels of known size: dst[i] = src[i] over `bytes` (multiple of 16; reads and
 * writes `bytes` each), and a read-only pass that folds `bytes` of src into 8 bytes at sink.
 * They give the memory system's practical rate and the reference dispatches that the
 * FETCH_SIZE / WRITE_SIZE counters are scaled by. */
int ozp_launch_copy(void* stream, void* dst, const void* src, size_t bytes);
int ozp_launch_read(void* stream, const void* src, size_t bytes, void* sink);

#ifdef __cplusplus
}
#endif
#endif /* OZPROBE_H */
