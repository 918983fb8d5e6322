"""The vendor baseline that the measurement tools report (hipSPARSE through paper_2511_17594_amd/vendor.py)
computes the same quantities as the library: C = A B and out[p] = <X_i, Y_j> on the same device buffers.
Both are compared with the oracle, so a wrong descriptor (layout, transpose flag, index type) cannot pass
for a slow vendor kernel."""
import numpy as np
import pytest

import oracle
from paper_2511_17594_amd import workloads as W
from util import dev, rel_l1_rows, rel_l1_segments

pytestmark = pytest.mark.gpu


def test_vendor_spmm_and_sddmm_match_the_oracle():
    import torch
    from paper_2511_17594_amd import vendor
    try:
        vs = vendor.Session(torch)
    except vendor.VendorError as e:
        pytest.skip("hipSPARSE not available: %s" % e)
    A, F = W.config1_tiny()[0], 32
    rng = np.random.default_rng(9)
    B = rng.standard_normal((A.n_cols, F)).astype(np.float32)
    X = rng.standard_normal((A.n_rows, F)).astype(np.float32)
    rp, ci, va, dB, dX = (dev(t, torch) for t in (A.rowptr, A.colind, A.val, B, X))
    ref_c = oracle.spmm(A.rowptr, A.colind, A.val, B)
    abs_c = oracle.spmm(A.rowptr, A.colind, np.abs(A.val), np.abs(B))
    ref_s = oracle.sddmm(A.rowptr, A.colind, X, B)
    abs_s = oracle.sddmm(A.rowptr, A.colind, np.abs(X), np.abs(B))
    try:
        for name, alg in vendor.SPMM_ALGS.items():
            C = torch.full((A.n_rows, F), float("nan"), device="cuda")
            t = vs.spmm_times(A.n_rows, A.n_cols, rp, ci, va, dB, C, iters=1, algs={name: alg})
            if not t:
                continue                                         # the library refuses this algorithm for the shape
            torch.cuda.synchronize()
            assert t[name] > 0 and rel_l1_rows(C.cpu().numpy(), ref_c, abs_c, terms=A.degrees).max() <= 1e-5, name
        out = torch.zeros(A.nnz, device="cuda")                  # the vendor SDDMM forms beta * out with beta = 0: no NaN in it
        t = vs.sddmm_time(A.n_rows, A.n_cols, rp, ci, dX, dB, out, iters=1)
        if t is not None:
            torch.cuda.synchronize()
            assert rel_l1_segments(out.cpu().numpy(), ref_s, A.rowptr, abs_s, terms=F).max() <= 1e-5
    finally:
        vs.close()
