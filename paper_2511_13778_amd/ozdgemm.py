"""Thin ctypes binding of the C-ABI library (include/ozdgemm.h): argument marshalling only.

Every step of the path runs in the HIP kernels behind the ABI.  PyTorch is used for device
memory and streams.  There is no CPU fallback: if the compiled library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liboz_mi355x.so")

OZ_DYNAMIC, OZ_FORCED_GUARDED, OZ_FIXED_GUARDED, OZ_FIXED_UNGUARDED, OZ_NATIVE = range(5)
OZ_NUM_STAGES = 7
OZ_STATIC_SCRATCH_BYTES = 256 << 20
STAGE_NAMES = ("scan", "esc", "verdict", "slicing", "slice_gemm_i8", "recompose", "native_dgemm")
STATUS = {0: "ok", 1: "invalid argument", 2: "workspace", 3: "device", 4: "hip"}


class oz_opts_t(C.Structure):
    _fields_ = [("mode", C.c_int32), ("target_bits", C.c_int32), ("max_bits", C.c_int32),
                ("slices", C.c_int32), ("esc_block", C.c_int32), ("heuristic", C.c_int32),
                ("tile_slices", C.c_int32)]


class oz_result_t(C.Structure):
    _fields_ = [("fallback", C.c_int32), ("reason", C.c_int32), ("slices_used", C.c_int32),
                ("esc", C.c_int32), ("required_bits", C.c_int32), ("infnan", C.c_int32),
                ("slices_min", C.c_int32), ("reserved_", C.c_int32), ("pair_tiles", C.c_int64)]


RESULT_INT32_WORDS = 10     # sizeof(oz_result_t) / 4


class oz_heuristic_t(C.Structure):
    _fields_ = [("int8_ops_per_ns", C.c_int64), ("fp64_flops_per_ns", C.c_int64),
                ("bytes_per_ns", C.c_int64), ("fixed_ns", C.c_int64)]


class oz_layout_t(C.Structure):
    _fields_ = [("mp", C.c_int64), ("np", C.c_int64), ("kp", C.c_int64), ("s_cap", C.c_int64),
                ("nkb", C.c_int64), ("kblk", C.c_int64),
                ("off_eA", C.c_size_t), ("off_eB", C.c_size_t), ("off_As", C.c_size_t),
                ("off_Bs", C.c_size_t), ("off_T", C.c_size_t), ("off_L", C.c_size_t),
                ("off_record", C.c_size_t), ("off_tileS", C.c_size_t), ("total_bytes", C.c_size_t)]


EXPORTS = ("oz_create", "oz_destroy", "oz_default_opts", "oz_set_heuristic",
           "oz_dgemm_workspace_bytes", "oz_dgemm", "oz_dgemm_static", "oz_zgemm_workspace_bytes", "oz_zgemm", "oz_dgemm_strided_batched", "oz_dgemm_layout", "oz_profile_enable",
           "oz_profile_read", "oz_native_dgemm", "oz_status_string")

_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2511_13778_amd.build` "
                           "(there is no CPU fallback)" % LIB_PATH)
    try:
        # torch ships its own HIP runtime; loading it first makes this library bind to the same copy
        # (two runtimes in one process do not both see the GPU)
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    H = C.c_void_p
    lib.oz_create.argtypes = [C.POINTER(H), C.c_int]
    lib.oz_create.restype = C.c_int
    lib.oz_destroy.argtypes = [H]
    lib.oz_destroy.restype = C.c_int
    lib.oz_default_opts.argtypes = [C.POINTER(oz_opts_t)]
    lib.oz_default_opts.restype = None
    lib.oz_set_heuristic.argtypes = [H, C.POINTER(oz_heuristic_t)]
    lib.oz_set_heuristic.restype = C.c_int
    dims = [C.c_char, C.c_char, C.c_int64, C.c_int64, C.c_int64]
    lib.oz_dgemm_workspace_bytes.argtypes = [H] + dims + [C.POINTER(oz_opts_t)]
    lib.oz_dgemm_workspace_bytes.restype = C.c_size_t
    lib.oz_dgemm_layout.argtypes = [H] + dims + [C.POINTER(oz_opts_t), C.POINTER(oz_layout_t)]
    lib.oz_dgemm_layout.restype = C.c_int
    gemm_args = [C.c_double, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_double, C.c_void_p, C.c_int64]
    lib.oz_dgemm.argtypes = [H, C.c_void_p] + dims + gemm_args + [C.POINTER(oz_opts_t), C.c_void_p,
                                                                    C.c_size_t, C.c_void_p]
    lib.oz_dgemm.restype = C.c_int
    lib.oz_dgemm_static.argtypes = [H, C.c_void_p] + dims + gemm_args + [C.POINTER(oz_opts_t), C.c_void_p]
    lib.oz_dgemm_static.restype = C.c_int
    lib.oz_zgemm_workspace_bytes.argtypes = [H] + dims + [C.POINTER(oz_opts_t)]
    lib.oz_zgemm_workspace_bytes.restype = C.c_size_t
    lib.oz_zgemm.argtypes = [H, C.c_void_p] + dims + [C.POINTER(C.c_double), C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                                       C.POINTER(C.c_double), C.c_void_p, C.c_int64, C.POINTER(oz_opts_t),
                                                       C.c_void_p, C.c_size_t, C.c_void_p]
    lib.oz_zgemm.restype = C.c_int
    lib.oz_dgemm_strided_batched.argtypes = [H, C.c_void_p] + dims + [
        C.c_double, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_int64, C.c_double, C.c_void_p,
        C.c_int64, C.c_int64, C.c_int64, C.POINTER(oz_opts_t), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.oz_dgemm_strided_batched.restype = C.c_int
    lib.oz_native_dgemm.argtypes = [H, C.c_void_p] + dims + gemm_args
    lib.oz_native_dgemm.restype = C.c_int
    lib.oz_profile_enable.argtypes = [H, C.c_int32]
    lib.oz_profile_enable.restype = C.c_int
    lib.oz_profile_read.argtypes = [H, C.c_int32, C.POINTER(C.c_float)]
    lib.oz_profile_read.restype = C.c_int
    lib.oz_status_string.argtypes = [C.c_int]
    lib.oz_status_string.restype = C.c_char_p
    _lib = lib
    return lib


class OzError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__("%s failed: %s (status %d)" % (what, STATUS.get(status, "?"), status))
        self.status = status


def _check(status: int, what: str):
    if status != 0:
        raise OzError(status, what)


def make_opts(mode=OZ_DYNAMIC, target_bits=53, max_bits=200, slices=0, esc_block=0, heuristic=1,
              tile_slices=0) -> oz_opts_t:
    return oz_opts_t(mode, target_bits, max_bits, slices, esc_block, heuristic, tile_slices)


def default_opts() -> oz_opts_t:
    """The library's own defaults (oz_default_opts)."""
    o = oz_opts_t()
    load_library().oz_default_opts(C.byref(o))
    return o


def result_from_words(words) -> "Result":
    """oz_result_t from its ten int32 words (little-endian int64 in the last two)."""
    w = [int(v) for v in words]
    return Result(w[0], w[1], w[2], w[3], w[4], w[5], w[6], (w[8] & 0xFFFFFFFF) | (w[9] << 32))


@dataclass
class Result:
    fallback: int
    reason: int
    slices_used: int
    esc: int
    required_bits: int
    infnan: int
    slices_min: int = 0
    pair_tiles: int = 0


class Handle:
    """oz_create / oz_destroy wrapper.  All tensors passed in are torch CUDA tensors; the matrices
    are interpreted as column-major storage with the given leading dimensions."""

    def __init__(self, device: int = 0):
        self.lib = load_library()
        self._h = C.c_void_p()
        _check(self.lib.oz_create(C.byref(self._h), device), "oz_create")

    def close(self):
        if self._h:
            self.lib.oz_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_heuristic(self, int8_ops_per_ns, fp64_flops_per_ns, bytes_per_ns, fixed_ns):
        m = oz_heuristic_t(int8_ops_per_ns, fp64_flops_per_ns, bytes_per_ns, fixed_ns)
        _check(self.lib.oz_set_heuristic(self._h, C.byref(m)), "oz_set_heuristic")

    def workspace_bytes(self, transa, transb, m, n, k, opts: oz_opts_t) -> int:
        return int(self.lib.oz_dgemm_workspace_bytes(self._h, transa.encode(), transb.encode(), m, n, k,
                                                     C.byref(opts)))

    def layout(self, transa, transb, m, n, k, opts: oz_opts_t) -> oz_layout_t:
        L = oz_layout_t()
        _check(self.lib.oz_dgemm_layout(self._h, transa.encode(), transb.encode(), m, n, k, C.byref(opts),
                                        C.byref(L)), "oz_dgemm_layout")
        return L

    def dgemm(self, stream_ptr, transa, transb, m, n, k, alpha, A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc,
              opts: oz_opts_t, ws_ptr, ws_bytes, result_ptr=None):
        _check(self.lib.oz_dgemm(self._h, stream_ptr, transa.encode(), transb.encode(), m, n, k, alpha,
                                 A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc, C.byref(opts), ws_ptr, ws_bytes,
                                 result_ptr), "oz_dgemm")

    def dgemm_static(self, stream_ptr, transa, transb, m, n, k, alpha, A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc,
                     opts: oz_opts_t, result_ptr=None):
        _check(self.lib.oz_dgemm_static(self._h, stream_ptr, transa.encode(), transb.encode(), m, n, k, alpha,
                                        A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc, C.byref(opts), result_ptr),
               "oz_dgemm_static")

    def zgemm_workspace_bytes(self, transa, transb, m, n, k, opts: oz_opts_t) -> int:
        return int(self.lib.oz_zgemm_workspace_bytes(self._h, transa.encode(), transb.encode(), m, n, k, C.byref(opts)))

    def zgemm(self, stream_ptr, transa, transb, m, n, k, alpha: complex, A_ptr, lda, B_ptr, ldb, beta: complex, C_ptr,
              ldc, opts: oz_opts_t, ws_ptr, ws_bytes, results_ptr=None):
        al = (C.c_double * 2)(complex(alpha).real, complex(alpha).imag)
        be = (C.c_double * 2)(complex(beta).real, complex(beta).imag)
        _check(self.lib.oz_zgemm(self._h, stream_ptr, transa.encode(), transb.encode(), m, n, k, al, A_ptr, lda, B_ptr,
                                 ldb, be, C_ptr, ldc, C.byref(opts), ws_ptr, ws_bytes, results_ptr), "oz_zgemm")

    def dgemm_strided_batched(self, stream_ptr, transa, transb, m, n, k, alpha, A_ptr, lda, stride_a, B_ptr, ldb,
                              stride_b, beta, C_ptr, ldc, stride_c, batch_count, opts: oz_opts_t, ws_ptr, ws_bytes,
                              results_ptr=None):
        _check(self.lib.oz_dgemm_strided_batched(self._h, stream_ptr, transa.encode(), transb.encode(), m, n, k,
                                                 alpha, A_ptr, lda, stride_a, B_ptr, ldb, stride_b, beta, C_ptr,
                                                 ldc, stride_c, batch_count, C.byref(opts), ws_ptr, ws_bytes,
                                                 results_ptr), "oz_dgemm_strided_batched")

    def native_dgemm(self, stream_ptr, transa, transb, m, n, k, alpha, A_ptr, lda, B_ptr, ldb, beta, C_ptr,
                     ldc):
        _check(self.lib.oz_native_dgemm(self._h, stream_ptr, transa.encode(), transb.encode(), m, n, k,
                                        alpha, A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc), "oz_native_dgemm")

    def profile_enable(self, max_calls: int):
        _check(self.lib.oz_profile_enable(self._h, max_calls), "oz_profile_enable")

    def profile_read(self, call: int):
        buf = (C.c_float * OZ_NUM_STAGES)()
        _check(self.lib.oz_profile_read(self._h, call, buf), "oz_profile_read")
        return list(buf)


# ---- convenience layer over torch tensors (memory and streams only) ------------------------
def to_colmajor(x_np):
    """Device copy of a numpy matrix in column-major storage: a (cols, rows) row-major tensor."""
    import numpy as np
    import torch
    return torch.from_numpy(np.ascontiguousarray(np.asarray(x_np, dtype=np.float64).T)).cuda()


def from_colmajor(t):
    """Numpy (rows, cols) view of a column-major device matrix stored as a (cols, rows) tensor."""
    return t.cpu().numpy().T


class Gemm:
    """One problem shape bound to a workspace; call run() repeatedly."""

    def __init__(self, handle: Handle, m, n, k, opts: oz_opts_t, transa="N", transb="N"):
        import torch
        self.h, self.m, self.n, self.k, self.opts = handle, m, n, k, opts
        self.transa, self.transb = transa, transb
        self.ws_bytes = handle.workspace_bytes(transa, transb, m, n, k, opts)
        if self.ws_bytes == 0 and m > 0 and n > 0:
            raise OzError(1, "oz_dgemm_workspace_bytes")
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device="cuda")
        assert self.ws.data_ptr() % 256 == 0
        self.result_dev = torch.zeros(RESULT_INT32_WORDS, dtype=torch.int32, device="cuda")
        self.L = handle.layout(transa, transb, m, n, k, opts)

    def run(self, A, lda, B, ldb, Cm, ldc, alpha=1.0, beta=0.0):
        import torch
        st = torch.cuda.current_stream().cuda_stream
        self.h.dgemm(st, self.transa, self.transb, self.m, self.n, self.k, alpha, A.data_ptr(), lda,
                     B.data_ptr(), ldb, beta, Cm.data_ptr(), ldc, self.opts, self.ws.data_ptr(),
                     self.ws_bytes, self.result_dev.data_ptr())

    def result(self) -> Result:
        return result_from_words(self.result_dev.cpu().tolist())

    def tile_slice_counts(self):
        """Slice count of every 256 x 256 block of C, numpy (mp/256) x (np/256), block (ti, tj) at [ti, tj]
        (meaningful after a call in OZ_DYNAMIC mode with tile_slices)."""
        import torch
        L = self.L
        nti, ntj = L.mp // 256, L.np // 256
        return self._view(L.off_tileS, nti * ntj * 4, torch.int32).view(ntj, nti).cpu().numpy().T.copy()

    def tile_order(self):
        """The order in which the slice GEMM dealt the blocks of C to its workgroups in the last per-block call:
        entry p = index, in the GEMM's block order, of the block that ran at position p (stored behind the
        slice counts)."""
        import torch
        L = self.L
        tiles = (L.mp // 256) * (L.np // 256)
        return self._view(L.off_tileS + tiles * 4, tiles * 4, torch.int32).cpu().numpy().copy()

    # views of the intermediates in the workspace (for parity tests)
    def _view(self, off, nbytes, dtype):
        return self.ws[off:off + nbytes].view(dtype)

    def row_exponents(self):
        import torch
        L = self.L
        return (self._view(L.off_eA, L.mp * 4, torch.int32)[:self.m].cpu().numpy(),
                self._view(L.off_eB, L.np * 4, torch.int32)[:self.n].cpu().numpy())

    def slices(self, S):
        """(As, Bs) as numpy int8 arrays S x m x k and S x n x k."""
        import torch
        L = self.L
        out = []
        for off, rows_p, rows in ((L.off_As, L.mp, self.m), (L.off_Bs, L.np, self.n)):
            t = self._view(off, L.s_cap * L.kp * rows_p, torch.int8).view(L.s_cap, L.kp // 16, rows_p, 16)
            t = t[:S, :, :rows, :].permute(0, 2, 1, 3).reshape(S, rows, L.kp)[:, :, :self.k]
            out.append(t.cpu().numpy())
        return out

    def slices_sampled(self, S, rows, cols):
        """(As[:, rows, :], Bs[:, cols, :]) as numpy int8 arrays; the selection happens on the device."""
        import torch
        L = self.L
        out = []
        for off, rows_p, sel in ((L.off_As, L.mp, rows), (L.off_Bs, L.np, cols)):
            t = self._view(off, L.s_cap * L.kp * rows_p, torch.int8).view(L.s_cap, L.kp // 16, rows_p, 16)
            idx = torch.as_tensor(sel, device="cuda", dtype=torch.long)
            t = t[:S].index_select(2, idx).permute(0, 2, 1, 3).reshape(S, len(sel), L.kp)[:, :, :self.k]
            out.append(t.cpu().numpy())
        return out

    def _digit_views(self):
        import torch
        L = self.L
        T = self._view(L.off_T, L.nkb * L.np * L.mp * 4, torch.int32).view(L.nkb, L.np, L.mp)
        nd = max(L.s_cap - 1, 0)
        Lo = self._view(L.off_L, L.nkb * nd * L.np * L.mp, torch.int8).view(L.nkb, nd, L.np // 4, L.mp, 4)
        return T, Lo

    def digits_sampled(self, S, nkb, rows, cols):
        """Aggregated anti-diagonal sums restricted to rows x cols: (T nkb x len(rows) x len(cols) int32,
        lo nkb x (S-1) x len(rows) x len(cols) int8, lo[:, d-1] = digit of anti-diagonal d)."""
        import torch
        T, Lo = self._digit_views()
        ri = torch.as_tensor(rows, device="cuda", dtype=torch.long)
        ci = torch.as_tensor(cols, device="cuda", dtype=torch.long)
        t = T[:nkb].index_select(1, ci).index_select(2, ri).permute(0, 2, 1)
        lo = Lo[:nkb, :max(S - 1, 0)].index_select(3, ri).index_select(2, ci // 4)      # nkb, S-1, cols, rows, 4
        lo = torch.gather(lo, 4, (ci % 4).view(1, 1, -1, 1, 1).expand(lo.shape[0], lo.shape[1], -1, lo.shape[3], 1))
        return t.cpu().numpy(), lo.squeeze(4).permute(0, 1, 3, 2).cpu().numpy()

    def digits(self, S, nkb):
        """Aggregated anti-diagonal sums of the whole product: (T nkb x m x n int32, lo nkb x (S-1) x m x n int8)."""
        T, Lo = self._digit_views()
        L = self.L
        t = T[:nkb, :self.n, :self.m].permute(0, 2, 1)
        lo = Lo[:nkb, :max(S - 1, 0)].permute(0, 1, 3, 2, 4).reshape(nkb, max(S - 1, 0), L.mp, L.np)[:, :, :self.m, :self.n]
        return t.cpu().numpy(), lo.cpu().numpy()
