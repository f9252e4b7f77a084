"""oz_dgemm_static (the entry point that allocates nothing: its workspace is a static device array
inside the library) against oz_dgemm with a caller workspace, through the C ABI.

Two calls in a row share the array, the second with a smaller problem, so anything the second call
wrongly inherited from the first (stale slices, products, tables, counters) would show.  Bar: the
record and every element of C are identical to oz_dgemm's (the kernels are the same, the integer
steps are exact and the FP64 order is fixed), and C is bit-identical to the CPU oracle's.
"""
import numpy as np
import pytest

from oracle import ozaki as oz
from paper_2511_13778_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def test_static_workspace_entry_matches_oz_dgemm():
    from paper_2511_13778_amd import ozdgemm as g
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the HIP path cannot run (there is no CPU fallback)")
    h = g.Handle(0)
    st = torch.cuda.current_stream().cuda_stream
    opts = g.make_opts(mode=g.OZ_DYNAMIC, target_bits=53, max_bits=200, heuristic=0)
    try:
        for (m, n, k, phi, seed) in ((600, 520, 777, 1.0, 81), (130, 200, 260, 0.5, 82)):
            A, B, Cin = wl.lognormal_spread(m, k, n, phi, seed=seed, with_c=True)
            dA, dB = g.to_colmajor(A), g.to_colmajor(B)
            assert 0 < h.workspace_bytes("N", "N", m, n, k, opts) <= g.OZ_STATIC_SCRATCH_BYTES
            # reference: the existing entry point with a caller-owned workspace
            gm = g.Gemm(h, m, n, k, opts)
            dC_ref = g.to_colmajor(Cin)
            gm.run(dA, m, dB, k, dC_ref, m, 1.5, 0.5)
            torch.cuda.synchronize()
            ref = gm.result()
            # the call under test; outputs and the record buffer exist before the call
            dC = g.to_colmajor(Cin)
            rec = torch.full((g.RESULT_INT32_WORDS,), -7, dtype=torch.int32, device="cuda")
            torch.cuda.synchronize()
            h.dgemm_static(st, "N", "N", m, n, k, 1.5, dA.data_ptr(), m, dB.data_ptr(), k, 0.5, dC.data_ptr(), m,
                           opts, rec.data_ptr())
            torch.cuda.synchronize()
            got = g.result_from_words(rec.cpu().tolist())
            assert got == ref and got.fallback == 0 and got.slices_used >= 7
            assert torch.equal(dC, dC_ref)
            tr = oz.emulated_dgemm(A, B, 1.5, 0.5, Cin, mode=oz.MODE_DYNAMIC, target_bits=53, max_bits=200, keep=False)
            assert (got.slices_used, got.esc) == (tr.verdict.slices_used, tr.verdict.esc)
            np.testing.assert_array_equal(g.from_colmajor(dC), tr.C)
        # beyond the array's size: refused with a workspace error, nothing enqueued, C untouched
        big = g.make_opts(mode=g.OZ_FORCED_GUARDED, max_bits=55)
        assert h.workspace_bytes("N", "N", 4096, 4096, 4096, big) > g.OZ_STATIC_SCRATCH_BYTES
        d = torch.zeros(8, dtype=torch.float64, device="cuda")
        with pytest.raises(g.OzError) as e:
            h.dgemm_static(st, "N", "N", 4096, 4096, 4096, 1.0, d.data_ptr(), 4096, d.data_ptr(), 4096, 0.0,
                           d.data_ptr(), 4096, big, None)
        assert e.value.status == 2
        torch.cuda.synchronize()
    finally:
        h.close()
