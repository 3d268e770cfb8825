"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle finishes every one of these in seconds, so the comparison is
elementwise over the whole output:  |Y - Yref| <= 1e-5 * (|A| |X|).
Row-split kernels are skipped where a single 39 k-entry row would make them
take tens of milliseconds per launch for no extra coverage; the medium-size
tests run all four kernels on the same structure.
"""
import numpy as np
import pytest

import oracle
from paper_2106_16064_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-5
NAMES = {0: "rs_sr", 1: "rs_pr", 2: "nb_sr", 3: "nb_pr", -1: "auto"}


@pytest.fixture(scope="module")
def dg():
    from paper_2106_16064_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def rmat20():
    return wl.rmat_csr(20, 16, seed=0, values="uniform01")


@pytest.fixture(scope="module")
def stencil128():
    return wl.stencil27_csr(128, seed=0)


def run_cell(dg, A, X, algos):
    import torch
    N = X.shape[1]
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).cuda()
    for algo in algos:
        print(f"[case] {A.name} nnz={A.nnz} N={N} algo={NAMES[algo]}", flush=True)
        dY = torch.full((A.M, N), float("nan"), device="cuda:0")
        dA.spmm(dX, algo=algo, Y=dY)
        torch.cuda.synchronize()
        Y = dY.cpu().numpy()
        del dY
        assert not np.isnan(Y).any()
        ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
        assert ok, f"{NAMES[algo]} on {A.name} N={N}: worst |err|/bound {worst:.3e}"
    # properties that hold at any size: empty rows are exact zeros
    lens = A.row_lengths()
    assert np.all(Y[lens == 0] == 0.0)


def test_power_law_spmv(dg, rmat20):
    run_cell(dg, rmat20, wl.dense_matrix(rmat20.K, 1, "uniform", seed=0), (-1, 3, 2, 1, 0))


@pytest.mark.parametrize("N", [32, 64, 128])
def test_gnn_spmm(dg, rmat20, N):
    A = wl.CsrMatrix(rmat20.M, rmat20.K, rmat20.rowptr, rmat20.colidx,
                     (1.0 / np.repeat(rmat20.row_lengths(), rmat20.row_lengths())).astype(np.float32),
                     "rmat20_rownorm")
    run_cell(dg, A, wl.dense_matrix(A.K, N, "normal", seed=0), (-1, 2, 3) if N > 32 else (-1, 2, 3, 0))


@pytest.mark.parametrize("N", [1, 2, 4, 8])
def test_stencil(dg, stencil128, N):
    run_cell(dg, stencil128, wl.dense_matrix(stencil128.K, N, "uniform", seed=0), (-1, 0, 1, 2, 3))
    if N == 1:
        # closed form at full size: A(ones) * ones counts neighbours
        import torch
        ones = wl.stencil27_csr(128, values="ones")
        dA = dg.DeviceCsr(ones)
        Y = dA.spmm(torch.ones((ones.K, 1), device="cuda:0"), algo=3).cpu().numpy()[:, 0]
        assert np.array_equal(Y, ones.row_lengths().astype(np.float32)) and Y.astype(np.float64).sum() == (3 * 128 - 2) ** 3


@pytest.mark.parametrize("dist", wl.SWEEP_DISTS)
@pytest.mark.parametrize("mean,N", [(64, 1), (64, 32), (16, 4), (4, 512)])
def test_selector_sweep_matrices_at_full_size(dg, dist, mean, N):
    """The sweep's matrices (2^18 rows, four row-length laws) at their real size: every kernel and
    the adaptive call, elementwise against the oracle.  Row-split kernels are left out where one
    very long row would make them take tens of milliseconds for no extra coverage."""
    A = wl.sweep_csr(1 << 18, mean, dist, seed=1)
    heavy = A.row_lengths().max() > 2000
    run_cell(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=N), (-1, 2, 3) if heavy else (-1, 0, 1, 2, 3))
