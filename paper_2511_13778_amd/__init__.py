"""MI355X-native emulated DGEMM (Ozaki scheme I on INT8 MFMA, guarded by ESC/ADP).

The compute path lives in csrc/ (HIP kernels behind a C-ABI library); `ozdgemm` is the thin
ctypes binding.  Nothing is imported eagerly so that the input generators can be used without
the compiled library."""
