"""The entry point that allocates nothing: ``dgsp_features_from_csr_device_noalloc`` keeps its 64 bytes of
scratch in a static device array of the library instead of a caller workspace.

Called through the raw C-ABI (ctypes on ``libdgsp.so``) and compared with the workspace version
``dgsp_features_from_csr_device`` field by field - all sums are integer sums, so the bar is equality - on
two calls in a row, the second on a smaller matrix (the array keeps the first call's contents until the
library clears it), then once more on the first matrix, and against the oracle's own row statistics.
"""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2106_16064_amd import workloads as wl

pytestmark = pytest.mark.gpu
FIELDS = ("M", "K", "nnz", "max_row", "min_row", "avg_row", "stdv_row", "cv_row", "col_span")


def test_static_scratch_statistics_equal_the_workspace_version():
    import torch
    from paper_2106_16064_amd import binding as dg
    L = dg.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    big = wl.rmat_csr(scale=15, avg_degree=16, seed=11)                 # long and empty rows, 2^15 rows
    small = wl.poisson_csr(700, 900, 5.0, seed=12)                      # fewer rows, smaller sums, smaller maximum
    assert small.M < big.M and small.row_lengths().max() < big.row_lengths().max()
    workspace = torch.empty(dg.FEATURES_WORKSPACE_BYTES // 8, dtype=torch.int64, device="cuda:0")

    def both(A, with_columns=True):
        rp = torch.from_numpy(A.rowptr).cuda()
        ci = torch.from_numpy(A.colidx).cuda()
        cptr = ci.data_ptr() if with_columns else None
        print(f"[case] noalloc features {A.name} M={A.M} nnz={A.nnz} columns={with_columns}", flush=True)
        got, want = dg.Features(), dg.Features()
        rc = L.dgsp_features_from_csr_device_noalloc(A.M, A.K, rp.data_ptr(), cptr, ctypes.byref(got), stream)
        assert rc == dg.OK
        rc = L.dgsp_features_from_csr_device(A.M, A.K, rp.data_ptr(), cptr, workspace.data_ptr(), ctypes.byref(want),
                                             stream)
        assert rc == dg.OK
        for name in FIELDS:
            assert getattr(got, name) == getattr(want, name), (A.name, name)
        ref = oracle.row_features(A.rowptr)
        assert (got.nnz, got.max_row, got.min_row) == (ref["nnz"], ref["max_row"], ref["min_row"])
        assert got.avg_row == pytest.approx(ref["avg_row"], rel=1e-12)
        assert got.stdv_row == pytest.approx(ref["stdv_row"], rel=1e-9, abs=1e-12)
        return got

    first = both(big)
    second = both(small)                      # right after, smaller: nothing of the first call may be left
    assert second.max_row < first.max_row and second.nnz < first.nnz
    both(small, with_columns=False)           # col_span stays 0 without columns, whatever the array held
    again = both(big)
    for name in FIELDS:
        assert getattr(again, name) == getattr(first, name), name

    # limits and argument errors: nothing is enqueued, the status says so
    out = dg.Features()
    rp = torch.from_numpy(small.rowptr).cuda()
    too_many = (1 << 31) - 4096 + 1
    assert L.dgsp_features_from_csr_device_noalloc(too_many, 10, rp.data_ptr(), None, ctypes.byref(out), stream) == dg.ERR_INVALID_ARG
    assert L.dgsp_features_from_csr_device_noalloc(-1, 10, rp.data_ptr(), None, ctypes.byref(out), stream) == dg.ERR_INVALID_ARG
    assert L.dgsp_features_from_csr_device_noalloc(small.M, small.K, None, None, ctypes.byref(out), stream) == dg.ERR_INVALID_ARG
    assert L.dgsp_features_from_csr_device_noalloc(small.M, small.K, rp.data_ptr(), None, None, stream) == dg.ERR_INVALID_ARG
    assert L.dgsp_features_from_csr_device_noalloc(0, 5, None, None, ctypes.byref(out), stream) == dg.OK
    assert (out.M, out.K, out.nnz) == (0, 5, 0)
