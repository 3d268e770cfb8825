"""``Y = A X`` as a differentiable PyTorch operation (A fixed, X learnable).

The paper names graph neural networks as the user of its kernels (Section 1,
Section 5) and describes the forward product only.  The gradient with respect
to X is again a sparse x dense product, with the transposed matrix:
``dL/dX = A^T dL/dY``.  The transposed CSR arrays are built once per matrix on
the host (a counting sort by column, plain numpy) and live on the device next
to A; both products run through the same C-ABI kernels and selection rules.
The stored values of A get no gradient.
"""
from __future__ import annotations

import numpy as np

from . import binding as dg
from .workloads import CsrMatrix


def transpose_csr(A: CsrMatrix) -> CsrMatrix:
    """CSR arrays of A^T (columns of each row ascending; duplicates kept as separate entries)."""
    lens = np.bincount(A.colidx, minlength=A.K).astype(np.int64)
    rowptr = np.zeros(A.K + 1, dtype=np.int64)
    np.cumsum(lens, out=rowptr[1:])
    order = np.argsort(A.colidx, kind="stable")            # entries grouped by column, original (row) order kept
    rows = np.repeat(np.arange(A.M, dtype=np.int64), A.row_lengths())
    return CsrMatrix(A.K, A.M, rowptr.astype(np.int32), rows[order].astype(np.int32),
                     A.vals[order].astype(np.float32), A.name + "^T", {})


def transpose_device_csr(A: "dg.DeviceCsr") -> "dg.DeviceCsr":
    """A^T of a matrix that lives on the GPU, built there with PyTorch's sort / bincount / cumsum (data
    movement only: set-up, not part of the product).  Same layout as ``transpose_csr``: entries grouped by
    column, rows ascending inside a group."""
    import torch
    lens = (A.rowptr[1:] - A.rowptr[:-1]).to(torch.int64)
    rows = torch.repeat_interleave(torch.arange(A.M, device=A.rowptr.device, dtype=torch.int64), lens)
    cols = A.colidx.to(torch.int64)
    order = torch.argsort(cols, stable=True)
    rowptr = torch.zeros(A.K + 1, dtype=torch.int64, device=A.rowptr.device)
    rowptr[1:] = torch.cumsum(torch.bincount(cols, minlength=A.K), 0)
    return dg.DeviceCsr.from_device(A.K, A.M, rowptr, rows[order], A.vals[order])


class SparseOperator:
    """A and A^T on the device; ``op(X)`` is differentiable with respect to X.  ``A`` is a host ``CsrMatrix``
    or a ``DeviceCsr`` (e.g. ``DeviceCsr.from_torch_sparse_csr``), whose transpose is then built on the GPU."""

    def __init__(self, A, device="cuda:0"):
        if isinstance(A, dg.DeviceCsr):
            self.fwd = A
            self.bwd = transpose_device_csr(A)
        else:
            self.fwd = dg.DeviceCsr(A, device)
            self.bwd = dg.DeviceCsr(transpose_csr(A), device)

    def __call__(self, X, algo=dg.AUTO):
        return _SpMM.apply(X, self, algo)


def _make_function():
    import torch

    class SpMM(torch.autograd.Function):
        @staticmethod
        def forward(ctx, X, op, algo):
            ctx.op = op
            squeeze = X.dim() == 1
            ctx.squeeze = squeeze
            Xc = (X.unsqueeze(1) if squeeze else X).contiguous().float()
            Y = op.fwd.spmm(Xc, algo=algo)
            return Y.squeeze(1) if squeeze else Y

        @staticmethod
        def backward(ctx, dY):
            G = (dY.unsqueeze(1) if ctx.squeeze else dY).contiguous().float()
            dX = ctx.op.bwd.spmm(G)           # the rules choose for A^T on their own
            return (dX.squeeze(1) if ctx.squeeze else dX), None, None

    return SpMM


class _Lazy:
    _fn = None

    @classmethod
    def apply(cls, *args):
        if cls._fn is None:
            cls._fn = _make_function()
        return cls._fn.apply(*args)


_SpMM = _Lazy
