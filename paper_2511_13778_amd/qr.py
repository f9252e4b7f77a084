"""Blocked Householder QR whose trailing-matrix update runs through oz_dgemm.

The paper's application experiment (section "Application-Level Integration", the blocked
Householder-QR algorithm with compact WY reflectors): the panel factorisation is left to the vendor
solver, the three matrix products of the trailing update

    W <- Y^T A_s,    W <- T^T W,    A_s <- A_s - Y W

are redirected to the emulated DGEMM with its guardrails.  Here the panel goes to torch.geqrf (the
vendor solver), T comes from the identity T^-1 + T^-T = Y^T Y for an orthogonal I - Y T Y^T (so
T^-1 = strict upper triangle of Y^T Y plus diag(1/tau)), and every product above is one oz_dgemm call
on sub-matrices of the column-major matrix: argument marshalling only, no arithmetic of the method
lives here.  Each call's device record is kept, so the driver can report which slice counts and
fallbacks the decision process chose over one factorisation, without a host-device synchronisation
inside the loop apart from what torch.geqrf does itself.
"""
from __future__ import annotations

from dataclasses import dataclass, field

from . import ozdgemm as g


@dataclass
class QrReport:
    records: list = field(default_factory=list)        # (m, n, k, Result) per oz_dgemm call
    panels: int = 0
    gemm_ms: float = 0.0                                # time of the trailing updates alone (HIP events)

    def histogram(self):
        """{label: number of GEMM calls}: 'S=<n>' for emulated calls (largest slice count of the call),
        'native:<reason>' for fallbacks."""
        names = {1: "inf/nan", 2: "bits", 3: "heuristic", 4: "forced"}
        out = {}
        for _, _, _, r in self.records:
            key = "native:%s" % names.get(r.reason, "?") if r.fallback else "S=%d" % r.slices_used
            out[key] = out.get(key, 0) + 1
        return out


def blocked_qr(handle: g.Handle, At, panel: int, opts: g.oz_opts_t):
    """In-place blocked Householder QR of the column-major m x n matrix stored in the torch CUDA tensor
    `At` of shape (n, m) (row j of At is column j of A; leading dimension m), m >= n, n a multiple of
    `panel`.  On return the upper triangle holds R and the part below the diagonal the Householder
    vectors, as LAPACK's geqrf leaves them.  Returns (tau, QrReport)."""
    import torch
    n, m = At.shape
    assert At.dtype == torch.float64 and At.is_cuda and At.is_contiguous() and m >= n and n % panel == 0
    b = panel
    st = torch.cuda.current_stream().cuda_stream
    steps = n // b
    # one workspace for the largest call of each kind (the first panel's), records for every call
    shapes = [("T", "N", b, n - b, m), ("T", "N", b, n - b, b), ("N", "N", m, n - b, b)] if steps > 1 else []
    ws_bytes = max([handle.workspace_bytes(ta, tb, mm, nn, kk, opts) for ta, tb, mm, nn, kk in shapes] + [256])
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    recs = torch.zeros((max(1, 3 * (steps - 1)), g.RESULT_INT32_WORDS), dtype=torch.int32, device="cuda")
    rec_bytes = 4 * g.RESULT_INT32_WORDS
    taus = torch.empty(n, dtype=torch.float64, device="cuda")
    Y = torch.empty((b, m), dtype=torch.float64, device="cuda")          # column-major rows x b, ld = rows
    W = torch.empty((n, b), dtype=torch.float64, device="cuda")          # column-major b x cols, ld = b
    W2 = torch.empty((n, b), dtype=torch.float64, device="cuda")
    eye = torch.eye(b, dtype=torch.float64, device="cuda")
    report = QrReport()
    call = 0
    marks = []
    for s in range(steps):
        c0, c1 = s * b, (s + 1) * b
        rows, cols = m - c0, n - c1
        # panel factorisation (vendor solver) on a copy of the rows x b panel, written back in place
        Pq, tau = torch.geqrf(At[c0:c1, c0:].T.contiguous())
        At[c0:c1, c0:] = Pq.T
        taus[c0:c1] = tau
        report.panels += 1
        if cols == 0:
            break
        # explicit Y (unit lower trapezoid) as a column-major rows x b matrix, and T from Y^T Y
        Yv = Y.view(-1)[: b * rows].view(b, rows)
        Yv.copy_(torch.tril(Pq, -1).T)
        Yv[:, :b] += eye
        G = Yv @ Yv.T
        Tinv = torch.triu(G, 1) + torch.diag(1.0 / tau)
        T = torch.linalg.solve_triangular(Tinv, eye, upper=True)         # b x b, upper triangular
        Tcm = T.T.contiguous()                                            # column-major storage of T
        As_ptr = At.data_ptr() + (c1 * m + c0) * 8                        # A_s = A[c0:, c1:], ld = m
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for (ta, tb, mm, nn, kk, alpha, A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc) in (
                ("T", "N", b, cols, rows, 1.0, Yv.data_ptr(), rows, As_ptr, m, 0.0, W.data_ptr(), b),
                ("T", "N", b, cols, b, 1.0, Tcm.data_ptr(), b, W.data_ptr(), b, 0.0, W2.data_ptr(), b),
                ("N", "N", rows, cols, b, -1.0, Yv.data_ptr(), rows, W2.data_ptr(), b, 1.0, As_ptr, m)):
            handle.dgemm(st, ta, tb, mm, nn, kk, alpha, A_ptr, lda, B_ptr, ldb, beta, C_ptr, ldc, opts,
                         ws.data_ptr(), ws_bytes, recs.data_ptr() + call * rec_bytes)
            report.records.append((mm, nn, kk, call))
            call += 1
        e1.record()
        marks.append((e0, e1))
    torch.cuda.synchronize()
    report.gemm_ms = float(sum(a.elapsed_time(b_) for a, b_ in marks))
    host = recs.cpu().tolist()
    report.records = [(mm, nn, kk, g.result_from_words(host[c])) for mm, nn, kk, c in report.records]
    return taus, report
