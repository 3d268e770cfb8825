"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle finishes every one of these in seconds, so the comparison is
elementwise over the whole output:  |Y - Yref| <= 1e-5 * (|A| |X|).
Every cell runs all four kernels and the adaptive call, also where a single
39 k-entry row makes a row-split kernel take tens of milliseconds.
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


@pytest.mark.parametrize("N", [2, 3, 4])
def test_power_law_narrow_spmm_plain_and_scaled(dg, rmat20, N):
    """The power-law matrix at two to four dense columns: sixteen million entries, so the balanced parallel kernel
    walks entry blocks at two, three and four columns per lane - in its plain form and in the scaled one
    (alpha A X + beta Y), which are separate instantiations."""
    import torch
    A = rmat20
    X = wl.dense_matrix(A.K, N, "uniform", seed=N)
    run_cell(dg, A, X, (3, -1))
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    Y0 = np.random.default_rng(N).uniform(-1.0, 1.0, size=(A.M, N)).astype(np.float32)
    alpha, beta = -2.0, 0.5
    want = alpha * yref + beta * Y0.astype(np.float64)
    bound = abs(alpha) * bnd + abs(beta) * np.abs(Y0.astype(np.float64))
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).cuda()
    for algo in (3, -1):
        print(f"[case] {A.name} N={N} scaled algo={NAMES[algo]}", flush=True)
        dY = torch.from_numpy(Y0).cuda()
        dg.dgsp_spmm_csr_axpby(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, alpha, beta, algo, dA.features)
        torch.cuda.synchronize()
        ok, worst = oracle.within_bound(dY.cpu().numpy(), want, bound, TOL)
        assert ok, f"scaled {NAMES[algo]} N={N}: worst |err|/bound {worst:.3e}"


@pytest.mark.parametrize("N", [32, 64, 128])
def test_gnn_spmm(dg, rmat20, N):
    A = wl.CsrMatrix(rmat20.M, rmat20.K, rmat20.rowptr, rmat20.colidx,
                     (1.0 / np.repeat(rmat20.row_lengths(), rmat20.row_lengths())).astype(np.float32),
                     "rmat20_rownorm")
    run_cell(dg, A, wl.dense_matrix(A.K, N, "normal", seed=0), (-1, 0, 1, 2, 3))


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
    the adaptive call, elementwise against the oracle."""
    A = wl.sweep_csr(1 << 18, mean, dist, seed=1)
    run_cell(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=N), (-1, 0, 1, 2, 3))


# ------------------------------------------------------------------ more than 2^30 stored entries
BIG_M = BIG_K = 1 << 20


def big_row_lengths(rows):
    return 1024 + (rows % 512)


def big_entries(rows):
    """Columns and values of the given rows of the 1.34e9-entry matrix, from its closed form:
    row i holds 1024 + i mod 512 entries; its j-th entry has column (977 i + 811 j) mod 2^20
    (distinct within a row, not ascending) and value ((40503 p) mod 65536) / 65536 - 1/2 with
    p the entry's position in the whole matrix.  Every step is exact in fp32 and in int64."""
    rows = np.asarray(rows, dtype=np.int64)
    lens = big_row_lengths(rows)
    starts = 1024 * rows + 512 * 511 // 2 * (rows // 512) + (rows % 512) * (rows % 512 - 1) // 2
    row_of = np.repeat(np.arange(rows.size), lens)
    j = np.arange(int(lens.sum()), dtype=np.int64) - np.repeat(np.cumsum(lens) - lens, lens)
    p = starts[row_of] + j
    col = (977 * rows[row_of] + 811 * j) % BIG_K
    val = ((40503 * p) % 65536).astype(np.float32) / np.float32(65536.0) - np.float32(0.5)
    return lens, col.astype(np.int32), val


def test_more_than_two_to_the_thirty_entries(dg):
    """1.34e9 stored entries: the column and value arrays pass 4 GB each, so entry positions no longer
    fit a 32-bit byte offset from the arrays' starts.  The matrix is written on the device from a
    closed form; the oracle recomputes sampled rows from the same form on the host - among them the
    rows around the 4 GB mark and the last ones."""
    import torch
    dev = torch.device("cuda:0")
    rows = torch.arange(BIG_M, dtype=torch.int64, device=dev)
    lens = 1024 + (rows % 512)
    rowptr64 = torch.zeros(BIG_M + 1, dtype=torch.int64, device=dev)
    rowptr64[1:] = torch.cumsum(lens, 0)
    nnz = int(rowptr64[-1])
    assert (1 << 30) < nnz < (1 << 31) - 4096
    rowptr = rowptr64.to(torch.int32)
    colidx = torch.empty(nnz, dtype=torch.int32, device=dev)
    vals = torch.empty(nnz, dtype=torch.float32, device=dev)
    step = 1 << 26
    for lo in range(0, nnz, step):
        p = torch.arange(lo, min(lo + step, nnz), dtype=torch.int64, device=dev)
        i = torch.searchsorted(rowptr64, p, right=True) - 1
        j = p - rowptr64[i]
        colidx[lo:lo + p.numel()] = ((977 * i + 811 * j) % BIG_K).to(torch.int32)
        vals[lo:lo + p.numel()] = ((40503 * p) % 65536).to(torch.float32) / 65536.0 - 0.5
    del p, i, j, rows, lens
    A = dg.DeviceCsr.from_device(BIG_M, BIG_K, rowptr, colidx, vals)
    assert A.nnz == nnz and A.features.max_row == 1535 and A.features.min_row == 1024

    # sampled rows: a seeded draw, the rows on both sides of byte 2^32 of the entry arrays, both ends
    rp = rowptr64.cpu().numpy()
    at_4g = int(np.searchsorted(rp, 1 << 30))
    sample = np.unique(np.concatenate([
        np.random.default_rng(5).integers(0, BIG_M, size=1500), np.arange(at_4g - 40, at_4g + 40),
        np.arange(0, 70), np.arange(BIG_M - 70, BIG_M)]))
    slens, scol, sval = big_entries(sample)
    assert np.array_equal(slens, np.diff(rp)[sample])
    # the device arrays hold what the closed form says (bit for bit) on the sampled rows
    first = sample[len(sample) // 2]
    a, b = int(rp[first]), int(rp[first + 1])
    l1, c1, v1 = big_entries([first])
    assert np.array_equal(colidx[a:b].cpu().numpy(), c1) and np.array_equal(vals[a:b].cpu().numpy(), v1)
    srowptr = np.zeros(sample.size + 1, dtype=np.int32)
    srowptr[1:] = np.cumsum(slens)

    for N, algos in ((1, (-1, 3, 2, 1, 0)), (4, (-1, 2, 0))):
        X = wl.dense_matrix(BIG_K, N, "uniform", seed=40 + N)
        yref, bnd = oracle.spmm_ref(sample.size, BIG_K, N, srowptr, scol, sval, X)
        dX = torch.from_numpy(X).cuda()
        for algo in algos:
            print(f"[case] 1.34e9 entries N={N} algo={NAMES[algo]}", flush=True)
            dY = torch.full((BIG_M, N), float("nan"), device=dev)
            A.spmm(dX, algo=algo, Y=dY)
            torch.cuda.synchronize()
            assert not bool(torch.isnan(dY).any())
            Y = dY[torch.from_numpy(sample).cuda()].cpu().numpy()
            ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
            assert ok, f"{NAMES[algo]} N={N}: worst |err|/bound {worst:.3e}"


# ------------------------------------------------------------------ 64-bit row pointers, more than 2^31 stored entries
def test_sixty_four_bit_row_pointers_small(dg):
    """dgsp_spmm_csr_i64 on matrices the other entry points take as well: the same products, every kernel."""
    import torch
    for A, N in ((wl.rmat_csr(scale=14, avg_degree=16, seed=51), 1), (wl.poisson_csr(3000, 2000, 9.0, seed=52), 4),
                 (wl.csr_from_lens(np.zeros(500, dtype=np.int64), 40, seed=53, name="no_entries"), 3)):
        X = wl.dense_matrix(A.K, N, "uniform", seed=54)
        yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
        rp = torch.from_numpy(A.rowptr.astype(np.int64)).cuda()
        ci, va = torch.from_numpy(A.colidx).cuda(), torch.from_numpy(A.vals).cuda()
        dX = torch.from_numpy(X).cuda()
        for algo in (-1, 0, 1, 2, 3):
            print(f"[case] i64 {A.name} N={N} algo={NAMES[algo]}", flush=True)
            dY = torch.full((A.M, N), float("nan"), device="cuda:0")
            dg.dgsp_spmm_csr_i64(A.M, A.K, N, A.nnz, rp, ci, va, dX, dY, algo)
            torch.cuda.synchronize()
            ok, worst = oracle.within_bound(dY.cpu().numpy(), yref, bnd, TOL)
            assert ok, f"{NAMES[algo]} on {A.name}: worst |err|/bound {worst:.3e}"
    # a wrong entry count, a short workspace and a 32-bit-style misuse are refused
    L = dg.lib()
    A = wl.poisson_csr(300, 200, 5.0, seed=55)
    rp = torch.from_numpy(A.rowptr.astype(np.int64)).cuda()
    ci, va = torch.from_numpy(A.colidx).cuda(), torch.from_numpy(A.vals).cuda()
    dX = torch.zeros((A.K, 1), device="cuda:0"); dY = torch.zeros((A.M, 1), device="cuda:0")
    big = torch.empty(1 << 16, dtype=torch.uint8, device="cuda:0")
    args = (rp.data_ptr(), ci.data_ptr(), va.data_ptr(), dX.data_ptr(), dY.data_ptr(), 3)
    assert L.dgsp_spmm_csr_i64(A.M, A.K, 1, A.nnz + 1, *args, big.data_ptr(), big.numel(), None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr_i64(A.M, A.K, 1, A.nnz, *args, big.data_ptr(), 64, None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr_i64(A.M, A.K, 1, A.nnz, *args, None, 1 << 16, None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr_i64(A.M, A.K, 1, -1, *args, big.data_ptr(), big.numel(), None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr_i64(A.M, A.K, 1, A.nnz, *args, big.data_ptr(), big.numel(), None) == dg.OK
    torch.cuda.synchronize()


def test_more_than_two_to_the_thirty_one_entries(dg):
    """2.68e9 stored entries behind 64-bit row pointers: entry positions pass 2^31, so the matrix is only reachable
    through dgsp_spmm_csr_i64, which cuts it into three slabs.  Built on the device from the closed form of
    big_entries(); the oracle recomputes sampled rows on the host - among them the rows on both sides of every slab
    cut (entry positions 2^30 and 2^31), around position 2^31 + 2^30 bytes apart, and both ends."""
    import torch
    dev = torch.device("cuda:0")
    M = 1 << 21
    rows = torch.arange(M, dtype=torch.int64, device=dev)
    lens = 1024 + (rows % 512)
    rowptr = torch.zeros(M + 1, dtype=torch.int64, device=dev)
    rowptr[1:] = torch.cumsum(lens, 0)
    nnz = int(rowptr[-1])
    assert nnz > (1 << 31)
    colidx = torch.empty(nnz, dtype=torch.int32, device=dev)
    vals = torch.empty(nnz, dtype=torch.float32, device=dev)
    step = 1 << 26
    for lo in range(0, nnz, step):
        p = torch.arange(lo, min(lo + step, nnz), dtype=torch.int64, device=dev)
        i = torch.searchsorted(rowptr, p, right=True) - 1
        j = p - rowptr[i]
        colidx[lo:lo + p.numel()] = ((977 * i + 811 * j) % BIG_K).to(torch.int32)
        vals[lo:lo + p.numel()] = ((40503 * p) % 65536).to(torch.float32) / 65536.0 - 0.5
    del p, i, j, rows, lens
    rp = rowptr.cpu().numpy()
    cuts = [int(np.searchsorted(rp, k << 30)) for k in (1, 2)]
    sample = np.unique(np.concatenate(
        [np.random.default_rng(6).integers(0, M, size=1200), np.arange(0, 66), np.arange(M - 66, M)]
        + [np.arange(c - 70, c + 70) for c in cuts]))
    slens, scol, sval = big_entries(sample)
    assert np.array_equal(slens, np.diff(rp)[sample])
    srowptr = np.zeros(sample.size + 1, dtype=np.int32)
    srowptr[1:] = np.cumsum(slens)
    workspace = torch.empty(dg.lib().dgsp_spmm_csr_i64_workspace_bytes(M, nnz), dtype=torch.uint8, device=dev)
    for N, algos in ((1, (-1, 3, 2, 1, 0)), (4, (2, 0))):
        X = wl.dense_matrix(BIG_K, N, "uniform", seed=60 + N)
        yref, bnd = oracle.spmm_ref(sample.size, BIG_K, N, srowptr, scol, sval, X)
        dX = torch.from_numpy(X).cuda()
        for algo in algos:
            print(f"[case] 2.68e9 entries (int64 row pointers) N={N} algo={NAMES[algo]}", flush=True)
            dY = torch.full((M, N), float("nan"), device=dev)
            dg.dgsp_spmm_csr_i64(M, BIG_K, N, nnz, rowptr, colidx, vals, dX, dY, algo, workspace)
            torch.cuda.synchronize()
            assert not bool(torch.isnan(dY).any())
            Y = dY[torch.from_numpy(sample).cuda()].cpu().numpy()
            ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
            assert ok, f"{NAMES[algo]} N={N}: worst |err|/bound {worst:.3e}"


# ------------------------------------------------------------------ dense operands beyond 4 GB
def test_dense_operands_beyond_four_gigabytes(dg, rmat20):
    """X and Y as column slices of 2^20 x 1100 buffers (4.6 GB each): byte offsets into them pass 2^32, so the
    kernels leave their 32-bit descriptor addressing for X and address Y rows with 64-bit arithmetic.  Widths 1, 4,
    8 and 5 (the shared-lane path); the balanced kernels on the R-MAT matrix, all four on a small Poisson matrix
    whose columns span all of K, the latter also in the scaled form."""
    import torch
    dev = torch.device("cuda:0")
    K = rmat20.K
    ld = 1100
    bigX = torch.empty((K, ld), dtype=torch.float32, device=dev)
    bigY = torch.empty((rmat20.M, ld), dtype=torch.float32, device=dev)
    assert bigX.numel() * 4 > (1 << 32)
    small = wl.csr_from_lens(np.random.default_rng(3).poisson(12.0, size=20000), K, seed=4, name="poisson12_wideK")
    cases = [(rmat20, (-1, 3, 2)), (small, (-1, 0, 1, 2, 3))]
    for N in (1, 4, 8, 5):
        x0, y0 = ld - N - 3, ld - N
        X = wl.dense_matrix(K, N, "uniform", seed=70 + N)
        bigX[:, x0:x0 + N] = torch.from_numpy(X).to(dev)
        for A, algos in cases:
            yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
            dA = dg.DeviceCsr(A)
            for algo in algos:
                print(f"[case] beyond 4 GB {A.name} N={N} algo={NAMES[algo]}", flush=True)
                bigY[:A.M, y0 - 2:] = float("nan")
                dg.dgsp_spmm_csr_ld(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, bigX[:, x0:x0 + N],
                                    bigY[:A.M, y0:y0 + N], algo, dA.features)
                torch.cuda.synchronize()
                out = bigY[:A.M, y0 - 2:].cpu().numpy()
                assert np.isnan(out[:, :2]).all(), "wrote left of the slice"
                Y = out[:, 2:]
                assert not np.isnan(Y).any()
                ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
                assert ok, f"{NAMES[algo]} on {A.name} N={N}: worst |err|/bound {worst:.3e}"
    # the scaled form on the same operands (N = 5 is still in place in bigX)
    N, alpha, beta = 5, 2.0, -0.5
    x0, y0 = ld - N - 3, ld - N
    yref, bnd = oracle.spmm_ref(small.M, small.K, N, small.rowptr, small.colidx, small.vals, X)
    Y0 = wl.dense_matrix(small.M, N, "uniform", seed=9)
    want = alpha * yref + beta * Y0.astype(np.float64)
    bound = abs(alpha) * bnd + abs(beta) * np.abs(Y0.astype(np.float64))
    dA = dg.DeviceCsr(small)
    for algo in (-1, 0, 1, 2, 3):
        print(f"[case] beyond 4 GB scaled N={N} algo={NAMES[algo]}", flush=True)
        bigY[:small.M, y0:y0 + N] = torch.from_numpy(Y0).to(dev)
        dg.dgsp_spmm_csr_axpby(small.M, small.K, N, small.nnz, dA.rowptr, dA.colidx, dA.vals, bigX[:, x0:x0 + N],
                               bigY[:small.M, y0:y0 + N], alpha, beta, algo, dA.features)
        torch.cuda.synchronize()
        ok, worst = oracle.within_bound(bigY[:small.M, y0:y0 + N].cpu().numpy(), want, bound, TOL)
        assert ok, f"scaled {NAMES[algo]}: worst |err|/bound {worst:.3e}"
