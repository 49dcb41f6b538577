"""The entry point for callers that cannot allocate: spqr_gemm_smallbatch_noalloc keeps its scratch in a static
device array.  Its output must equal spqr_gemm_smallbatch_ws's (same kernels, scratch elsewhere) bit for bit and
the oracle within tolerance, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

import spqr_synth as synth
from oracle import spqr_oracle as orc

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

REL_L2 = 1e-3


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def rel_l2(got, ref):
    return float(np.linalg.norm(np.asarray(got, np.float64) - ref) / np.linalg.norm(ref))


def test_static_scratch_entry_point_two_calls_in_a_row():
    import torch
    import paper_2306_03078_amd as P
    P.load_library()
    assert torch.cuda.is_available()
    P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_MATRIX)
    try:
        # first a large call (long outlier rows, several splits, a permutation), then a smaller one: the array
        # keeps the first call's contents
        big = synth.make_matrix(25 * 16, 300 * 16, w_bits=4, beta1=16, beta2=16, group_axis=1, outlier_rate=0.2,
                                outlier_structure="rows8cols4", seed=(61,))
        big.perm = np.random.default_rng(62).permutation(big.n).astype(np.int32)
        small = synth.make_matrix(5 * 8, 67 * 32, w_bits=3, beta1=8, beta2=32, group_axis=1, outlier_rate=0.03,
                                  outlier_structure="cols64", seed=(63,))
        for f, b in ((big, 16), (small, 7), (big, 37), (small, 16)):
            A = P.SpQRMatrix.from_logical(f)
            X = dev(synth.make_x(f.n, b, seed=(64, b)))
            need = P.spqr_workspace_bytes(A, b)
            assert 0 < need <= P.SPQR_STATIC_SCRATCH_BYTES
            ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
            want = P.spqr_gemm_smallbatch_ws(A, X, ws)
            for dt in (P.SPQR_F32, P.SPQR_F16):
                out = torch.zeros((b, f.m), dtype=torch.float32 if dt == P.SPQR_F32 else torch.float16, device="cuda:0")
                P.spqr_gemm_smallbatch_noalloc(A, X, out, y_dtype=dt)
                torch.cuda.synchronize()
                if dt == P.SPQR_F32:
                    assert torch.equal(out, want)
                    ref = orc.matvec(f, X.cpu().numpy())
                    assert max(rel_l2(out.cpu().numpy()[k], ref[k]) for k in range(b)) <= REL_L2
                else:
                    assert torch.equal(out, P.spqr_gemm_smallbatch_ws(A, X, ws, y_dtype=dt))
        # a batch the vector kernel takes needs no scratch and passes through as well
        A = P.SpQRMatrix.from_logical(small)
        X = dev(synth.make_x(small.n, 2, seed=(65,)))
        out = torch.zeros((2, small.m), dtype=torch.float32, device="cuda:0")
        P.spqr_gemm_smallbatch_noalloc(A, X, out)
        assert torch.equal(out, P.spqr_gemm_smallbatch(A, X))
        # beyond the static array: refused, nothing launched (a descriptor of a huge matrix; its pointers are never
        # followed because the size check comes first)
        huge = P.SpQRMatrix.from_logical(small)
        huge.desc.m, huge.desc.n = 16 * 65536, 32 * 64
        huge.desc.packed_bytes = P.packed_bytes(huge.desc.m, huge.desc.n, 3, 3, 3, 8, 32, 1)
        assert P.spqr_workspace_bytes(huge, 16) > P.SPQR_STATIC_SCRATCH_BYTES
        rc = P.load_library().spqr_gemm_smallbatch_noalloc(__import__("ctypes").byref(huge.desc), X.data_ptr(), 16,
                                                           out.data_ptr(), 0, None)
        assert rc == P.SPQR_ERR_WORKSPACE
    finally:
        P.spqr_set_option(P.SPQR_OPT_BATCH_PATH, P.SPQR_BATCH_PATH_AUTO)
