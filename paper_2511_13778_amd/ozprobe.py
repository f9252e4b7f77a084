"""ctypes binding of the measurement probes (include/ozprobe.h, liboz_probe.so): argument
marshalling only.  Used by bench.py to put the roofline fractions next to what the part sustains;
the product path (ozdgemm.py, liboz_mi355x.so) does not depend on it."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liboz_probe.so")
EXPORTS = ("ozp_launch_mfma_i8", "ozp_launch_copy", "ozp_launch_read")
MFMA_OPERAND_BYTES = 65536
MFMA_OPS_PER_WAVE_ITER = 16 * 65536          # 16 instructions of 32x32x32 multiply-adds, 2 ops each

_lib = None


def load_library() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_2511_13778_amd.build`" % LIB_PATH)
        try:
            import torch  # noqa: F401  (same HIP runtime as the tensors the probes are given)
        except ImportError:
            pass
        lib = C.CDLL(LIB_PATH)
        lib.ozp_launch_mfma_i8.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int]
        lib.ozp_launch_mfma_i8.restype = C.c_int
        lib.ozp_launch_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]
        lib.ozp_launch_copy.restype = C.c_int
        lib.ozp_launch_read.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.ozp_launch_read.restype = C.c_int
        _lib = lib
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError("%s failed with status %d" % (what, rc))


def launch_mfma_i8(stream_ptr, operands_ptr, sink_ptr, iters: int, workgroups: int):
    _check(load_library().ozp_launch_mfma_i8(stream_ptr, operands_ptr, sink_ptr, iters, workgroups), "ozp_launch_mfma_i8")


def launch_copy(stream_ptr, dst_ptr, src_ptr, nbytes: int):
    _check(load_library().ozp_launch_copy(stream_ptr, dst_ptr, src_ptr, nbytes), "ozp_launch_copy")


def launch_read(stream_ptr, src_ptr, nbytes: int, sink_ptr):
    _check(load_library().ozp_launch_read(stream_ptr, src_ptr, nbytes, sink_ptr), "ozp_launch_read")
