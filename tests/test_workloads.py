"""Structure and determinism of the seeded workload generators."""
import numpy as np
import pytest

from paper_2106_16064_amd import workloads as wl


def check_csr(A):
    assert A.rowptr.dtype == np.int32 and A.colidx.dtype == np.int32 and A.vals.dtype == np.float32
    assert A.rowptr.shape == (A.M + 1,) and A.rowptr[0] == 0
    assert np.all(np.diff(A.rowptr) >= 0)
    assert A.colidx.shape == (A.nnz,) and A.vals.shape == (A.nnz,)
    if A.nnz:
        assert A.colidx.min() >= 0 and A.colidx.max() < A.K
        rows = np.repeat(np.arange(A.M), A.row_lengths())
        key = rows.astype(np.int64) * A.K + A.colidx
        assert np.all(np.diff(key) > 0), "columns must be ascending and unique inside each row"
    assert np.all(np.isfinite(A.vals))


def test_poisson_tiny():
    A = wl.poisson_csr(4096, 4096, 8.0, seed=0)
    check_csr(A)
    s = A.stats()
    assert abs(s["mean"] - 8.0) < 0.2 and abs(s["std"] - np.sqrt(8.0)) < 0.2
    assert A.vals.min() >= -1 and A.vals.max() <= 1
    B = wl.poisson_csr(4096, 4096, 8.0, seed=0)
    assert np.array_equal(A.colidx, B.colidx) and np.array_equal(A.vals, B.vals)
    C = wl.poisson_csr(4096, 4096, 8.0, seed=1)
    assert not np.array_equal(A.rowptr, C.rowptr)


def test_rmat_small():
    A = wl.rmat_csr(scale=12, avg_degree=16, seed=0)
    check_csr(A)
    assert A.M == A.K == 4096
    assert A.nnz <= A.meta["edge_draws"]
    s = A.stats()
    assert s["cv"] > 1.5 and s["empty_frac"] > 0.05          # skewed, with empty rows
    assert A.vals.min() >= 0 and A.vals.max() < 1
    # quadrant a is the heaviest: most entries sit in the low-index corner
    assert (A.colidx < A.K // 2).mean() > 0.7
    B = wl.rmat_csr(scale=12, avg_degree=16, seed=0)
    assert np.array_equal(A.rowptr, B.rowptr) and np.array_equal(A.vals, B.vals)
    G = wl.rmat_csr(scale=12, avg_degree=16, seed=0, values="rownorm")
    assert np.array_equal(G.colidx, A.colidx)
    lens = np.repeat(G.row_lengths(), G.row_lengths())
    assert np.allclose(G.vals * lens, 1.0, rtol=1e-6)


@pytest.mark.parametrize("n", [3, 6])
def test_stencil(n):
    A = wl.stencil27_csr(n, seed=0)
    check_csr(A)
    assert A.nnz == (3 * n - 2) ** 3
    assert set(np.unique(A.row_lengths())) <= {8, 12, 18, 27}
    # diagonal entries carry the +27 shift
    rows = np.repeat(np.arange(A.M), A.row_lengths())
    d = A.vals[rows == A.colidx]
    assert d.size == A.M and d.mean() > 20


@pytest.mark.parametrize("dist", wl.SWEEP_DISTS)
@pytest.mark.parametrize("mean", [4, 16])
def test_sweep_means(dist, mean):
    A = wl.sweep_csr(1 << 14, mean, dist, seed=0)
    check_csr(A)
    s = A.stats()
    tol = 0.25 if dist in ("zipf", "lognormal") else 0.05
    assert abs(s["mean"] / mean - 1) < tol, s
    if dist == "fixed":
        assert s["std"] == 0
    if dist == "zipf":
        assert s["max"] <= wl.zipf_truncation(mean)


def test_zipf_truncation_points():
    assert wl.zipf_truncation(4) == 27
    assert wl.zipf_truncation(16) in (435, 436)
    assert wl.zipf_truncation(64) in (6982, 6983)


def test_distinct_columns_dense_rows():
    A = wl.csr_from_lens([0, 8, 3, 8, 1], K=8, seed=0)
    check_csr(A)
    assert list(A.row_lengths()) == [0, 8, 3, 8, 1]
    assert A.k_touched() == 8


def test_dense_matrix():
    X = wl.dense_matrix(100, 4, "uniform", seed=0)
    assert X.dtype == np.float32 and X.shape == (100, 4) and X.flags.c_contiguous
    assert np.array_equal(X, wl.dense_matrix(100, 4, "uniform", seed=0))
    assert abs(wl.dense_matrix(20000, 2, "normal", seed=0).std() - 1) < 0.02


def test_transposed_csr_is_the_transpose():
    """The arrays the backward product uses: compared with scipy's transpose on an unsorted matrix with duplicates."""
    import scipy.sparse as sp
    from paper_2106_16064_amd.autograd import transpose_csr
    rng = np.random.default_rng(5)
    M, K, nnz = 70, 45, 600
    rows = np.sort(rng.integers(0, M, size=nnz))
    cols = rng.integers(0, K, size=nnz).astype(np.int32)
    vals = rng.standard_normal(nnz).astype(np.float32)
    rowptr = np.zeros(M + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows, minlength=M), out=rowptr[1:])
    A = wl.CsrMatrix(M, K, rowptr, cols, vals, "t", {})
    T = transpose_csr(A)
    assert (T.M, T.K, T.nnz) == (K, M, nnz)
    assert T.rowptr[0] == 0 and np.all(np.diff(T.rowptr) >= 0) and T.rowptr[-1] == nnz
    want = sp.csr_matrix((vals.astype(np.float64), cols, rowptr), shape=(M, K)).T.toarray()
    got = sp.csr_matrix((T.vals.astype(np.float64), T.colidx, T.rowptr), shape=(K, M)).toarray()
    assert np.array_equal(got, want)
    for i in range(T.M):                                   # columns ascending inside every row of A^T
        assert np.all(np.diff(T.colidx[T.rowptr[i]:T.rowptr[i + 1]]) >= 0)
