"""Pins for the CPU oracle (paper Section 1: Y = A X).

None of these retypes the oracle's loop: they compare it with dense matmul, an
independent sparse library, a brute-force scatter over COO triples, algebraic
identities, a hand-worked fixture and closed forms on the benchmark
generators.  A dropped term, a sign slip, a transposed operand, an off-by-one
in the row range or a wrong leading dimension fails at least one of them.
"""
import os

import numpy as np
import pytest
import scipy.sparse as sp
from hypothesis import given, settings, strategies as st

import oracle
from paper_2106_16064_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_csr(rng, M, K, density, sort=True, dup=False):
    mask = rng.random((M, K)) < density
    rows, cols = np.nonzero(mask)
    if dup and rows.size:
        extra = rng.integers(0, rows.size, size=max(1, rows.size // 3))
        rows = np.concatenate([rows, rows[extra]])
        cols = np.concatenate([cols, cols[extra]])
    order = np.lexsort((cols, rows)) if sort else np.lexsort((rng.random(rows.size), rows))
    rows, cols = rows[order], cols[order]
    rowptr = np.zeros(M + 1, np.int32)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr).astype(np.int32)
    vals = rng.uniform(-1, 1, size=rows.size).astype(np.float32)
    return rowptr, cols.astype(np.int32), vals, rows


def densify(M, K, rowptr, colidx, vals):
    A = np.zeros((M, K), np.float64)
    for i in range(M):
        for p in range(rowptr[i], rowptr[i + 1]):
            A[i, colidx[p]] += float(vals[p])
    return A


# ---------------------------------------------------------------- fixture
def _read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            out[k] = np.array([float(t) for t in v])
    return out


def test_hand_worked_fixture():
    g = _read_golden(os.path.join(GOLDEN, "hand_worked_3x4.txt"))
    rowptr = g["rowptr"].astype(np.int32)
    colidx = g["colidx"].astype(np.int32)
    vals = g["vals"].astype(np.float32)
    X = g["X"].astype(np.float32).reshape(4, 2)
    for fn in (oracle.spmm_ref, oracle.spmm_ref_loops):
        y, b = fn(3, 4, 2, rowptr, colidx, vals, X)
        assert np.array_equal(y, g["Y"].reshape(3, 2))
        assert np.array_equal(b, g["B"].reshape(3, 2))


# ---------------------------------------------------------------- library / textbook reductions
@settings(max_examples=60, deadline=None)
@given(M=st.integers(1, 40), K=st.integers(1, 40), N=st.integers(1, 9),
       density=st.floats(0.0, 1.0), seed=st.integers(0, 2 ** 31 - 1),
       sort=st.booleans(), dup=st.booleans())
def test_against_dense_matmul(M, K, N, density, seed, sort, dup):
    rng = np.random.default_rng(seed)
    rowptr, colidx, vals, _ = random_csr(rng, M, K, density, sort, dup)
    X = rng.uniform(-1, 1, size=(K, N)).astype(np.float32)
    A = densify(M, K, rowptr, colidx, vals)
    want = A @ X.astype(np.float64)
    y, b = oracle.spmm_ref(M, K, N, rowptr, colidx, vals, X)
    scale = np.abs(A) @ np.abs(X.astype(np.float64)) + 1e-300
    assert np.all(np.abs(y - want) <= 1e-12 * scale)
    # the bound itself: |A| |X| with duplicates NOT merged before abs()
    Aabs = np.zeros((M, K))
    for i in range(M):
        for p in range(rowptr[i], rowptr[i + 1]):
            Aabs[i, colidx[p]] += abs(float(vals[p]))
    wantb = Aabs @ np.abs(X.astype(np.float64))
    assert np.allclose(b, wantb, rtol=1e-12, atol=0)
    assert np.all(b >= np.abs(y) * (1 - 1e-12))


@pytest.mark.parametrize("M,K,N,density", [(300, 170, 5, 0.05), (64, 512, 3, 0.2), (1000, 1000, 1, 0.01)])
def test_against_scipy(M, K, N, density):
    rng = np.random.default_rng(M + K + N)
    rowptr, colidx, vals, _ = random_csr(rng, M, K, density)
    X = rng.standard_normal((K, N)).astype(np.float32)
    A = sp.csr_matrix((vals.astype(np.float64), colidx, rowptr), shape=(M, K))
    want = A @ X.astype(np.float64)
    y = oracle.spmm_ref(M, K, N, rowptr, colidx, vals, X, with_bound=False)
    assert np.allclose(y, want, rtol=1e-12, atol=1e-13)


def test_brute_force_coo_scatter():
    rng = np.random.default_rng(7)
    M, K, N = 23, 31, 4
    rowptr, colidx, vals, rows = random_csr(rng, M, K, 0.3, sort=False, dup=True)
    X = rng.uniform(-1, 1, size=(K, N)).astype(np.float32)
    want = np.zeros((M, N))
    for i, k, v in zip(rows, colidx, vals):
        want[i, :] += float(v) * X[k, :].astype(np.float64)
    y = oracle.spmm_ref(M, K, N, rowptr, colidx, vals, X, with_bound=False)
    assert np.allclose(y, want, rtol=1e-13, atol=1e-15)


def test_c_oracle_equals_python_loops():
    rng = np.random.default_rng(11)
    for M, K, N in [(17, 9, 3), (5, 40, 7), (33, 33, 1)]:
        rowptr, colidx, vals, _ = random_csr(rng, M, K, 0.25, sort=False, dup=True)
        X = rng.standard_normal((K, N)).astype(np.float32)
        y1, b1 = oracle.spmm_ref(M, K, N, rowptr, colidx, vals, X)
        y2, b2 = oracle.spmm_ref_loops(M, K, N, rowptr, colidx, vals, X)
        assert np.array_equal(y1, y2) and np.array_equal(b1, b2)


def test_thread_count_does_not_change_bits():
    A = wl.poisson_csr(2000, 1500, 6.0, seed=3)
    X = wl.dense_matrix(A.K, 5, "normal", seed=3)
    y1 = oracle.spmm_ref(A.M, A.K, 5, A.rowptr, A.colidx, A.vals, X, with_bound=False, nthreads=1)
    y4 = oracle.spmm_ref(A.M, A.K, 5, A.rowptr, A.colidx, A.vals, X, with_bound=False, nthreads=4)
    assert np.array_equal(y1, y4)


# ---------------------------------------------------------------- invariants
def test_identity_returns_x_bit_exact():
    K, N = 50, 6
    rowptr = np.arange(K + 1, dtype=np.int32)
    colidx = np.arange(K, dtype=np.int32)
    vals = np.ones(K, np.float32)
    X = wl.dense_matrix(K, N, "normal", seed=1)
    y, b = oracle.spmm_ref(K, K, N, rowptr, colidx, vals, X)
    assert np.array_equal(y, X.astype(np.float64))
    assert np.array_equal(b, np.abs(X).astype(np.float64))


def test_permutation_matrix_gathers_rows():
    rng = np.random.default_rng(5)
    K, N = 37, 3
    perm = rng.permutation(K).astype(np.int32)
    X = wl.dense_matrix(K, N, "uniform", seed=2)
    y = oracle.spmm_ref(K, K, N, np.arange(K + 1, dtype=np.int32), perm, np.ones(K, np.float32), X,
                        with_bound=False)
    assert np.array_equal(y, X[perm].astype(np.float64))


def test_single_entry_row_and_empty_rows():
    M, K, N = 6, 8, 4
    rowptr = np.array([0, 0, 1, 1, 1, 2, 2], np.int32)
    colidx = np.array([5, 0], np.int32)
    vals = np.array([-0.75, 3.0], np.float32)
    X = wl.dense_matrix(K, N, "uniform", seed=4)
    y, b = oracle.spmm_ref(M, K, N, rowptr, colidx, vals, X)
    assert np.array_equal(y[1], -0.75 * X[5].astype(np.float64))
    assert np.array_equal(y[4], 3.0 * X[0].astype(np.float64))
    for r in (0, 2, 3, 5):
        assert np.all(y[r] == 0.0) and np.all(b[r] == 0.0)


def test_unit_vector_extracts_column_of_a():
    rng = np.random.default_rng(9)
    M, K = 30, 20
    rowptr, colidx, vals, _ = random_csr(rng, M, K, 0.3)
    A = densify(M, K, rowptr, colidx, vals)
    for j in (0, 7, K - 1):
        e = np.zeros((K, 1), np.float32)
        e[j] = 1.0
        y = oracle.spmm_ref(M, K, 1, rowptr, colidx, vals, e, with_bound=False)
        assert np.array_equal(y[:, 0], A[:, j])


def test_linearity_in_x():
    rng = np.random.default_rng(13)
    M, K, N = 40, 25, 3
    rowptr, colidx, vals, _ = random_csr(rng, M, K, 0.2)
    # dyadic X so that alpha*X1 + X2 is exact in fp32
    X1 = rng.integers(-8, 9, size=(K, N)).astype(np.float32) / 8
    X2 = rng.integers(-8, 9, size=(K, N)).astype(np.float32) / 4
    alpha = 0.5
    f = lambda X: oracle.spmm_ref(M, K, N, rowptr, colidx, vals, X, with_bound=False)
    lhs = f((alpha * X1 + X2).astype(np.float32))
    rhs = alpha * f(X1) + f(X2)
    assert np.allclose(lhs, rhs, rtol=1e-13, atol=1e-14)


def test_order_inside_row_and_duplicates():
    rng = np.random.default_rng(17)
    M, K, N = 12, 15, 2
    rowptr, colidx, vals, _ = random_csr(rng, M, K, 0.5)
    X = wl.dense_matrix(K, N, "normal", seed=6)
    y0 = oracle.spmm_ref(M, K, N, rowptr, colidx, vals, X, with_bound=False)
    c2, v2 = colidx.copy(), vals.copy()
    for i in range(M):
        s, e = rowptr[i], rowptr[i + 1]
        p = rng.permutation(e - s)
        c2[s:e], v2[s:e] = colidx[s:e][p], vals[s:e][p]
    y1 = oracle.spmm_ref(M, K, N, rowptr, c2, v2, X, with_bound=False)
    assert np.allclose(y0, y1, rtol=1e-13, atol=1e-15)
    # an entry split into two halves at the same (i,k) gives the same product
    rp = np.array([0, 2], np.int32)
    y_split = oracle.spmm_ref(1, K, N, rp, np.array([3, 3], np.int32), np.array([0.25, 0.5], np.float32), X,
                              with_bound=False)
    y_one = oracle.spmm_ref(1, K, N, np.array([0, 1], np.int32), np.array([3], np.int32),
                            np.array([0.75], np.float32), X, with_bound=False)
    assert np.array_equal(y_split, y_one)


def test_non_square_shapes_catch_transposes():
    # M, K, N pairwise different and X far from symmetric: reading X column-major
    # or swapping M and K changes the answer.
    M, K, N = 3, 5, 2
    rowptr = np.array([0, 1, 3, 4], np.int32)
    colidx = np.array([4, 0, 3, 1], np.int32)
    vals = np.array([1, 2, 4, 8], np.float32)
    X = np.arange(K * N, dtype=np.float32).reshape(K, N)  # X[k,n] = 2k+n
    y = oracle.spmm_ref(M, K, N, rowptr, colidx, vals, X, with_bound=False)
    want = np.array([[8, 9], [2 * 0 + 4 * 6, 2 * 1 + 4 * 7], [8 * 2, 8 * 3]], np.float64)
    assert np.array_equal(y, want)


def test_zero_extents():
    y, b = oracle.spmm_ref(0, 4, 3, np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                           np.zeros((4, 3), np.float32))
    assert y.shape == (0, 3)
    y = oracle.spmm_ref(3, 4, 2, np.zeros(4, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                        np.ones((4, 2), np.float32), with_bound=False)
    assert np.all(y == 0)


def test_rejects_malformed():
    X = np.ones((4, 1), np.float32)
    with pytest.raises(ValueError):
        oracle.spmm_ref(2, 4, 1, np.array([0, 2, 1], np.int32), np.array([0, 1], np.int32),
                        np.ones(2, np.float32), X)
    with pytest.raises(ValueError):
        oracle.spmm_ref(1, 4, 1, np.array([0, 1], np.int32), np.array([4], np.int32), np.ones(1, np.float32), X)


# ---------------------------------------------------------------- closed forms on the generators
def test_stencil_of_ones_counts_neighbours():
    n = 9
    A = wl.stencil27_csr(n, values="ones")
    ones = np.ones((A.K, 2), np.float32)
    y = oracle.spmm_ref(A.M, A.K, 2, A.rowptr, A.colidx, A.vals, ones, with_bound=False)
    idx = np.arange(n)
    per_dim = np.where((idx == 0) | (idx == n - 1), 2, 3)
    want = (per_dim[:, None, None] * per_dim[None, :, None] * per_dim[None, None, :]).ravel()
    assert np.array_equal(y[:, 0], want) and np.array_equal(y[:, 1], want)
    assert y[:, 0].sum() == (3 * n - 2) ** 3


def test_stencil_rowsum_matches_reduceat():
    A = wl.stencil27_csr(7, seed=2)
    ones = np.ones((A.K, 1), np.float32)
    y = oracle.spmm_ref(A.M, A.K, 1, A.rowptr, A.colidx, A.vals, ones, with_bound=False)
    want = np.add.reduceat(A.vals.astype(np.float64), A.rowptr[:-1].astype(np.int64))
    assert np.allclose(y[:, 0], want, rtol=1e-12, atol=1e-12)


def test_row_normalised_rmat_times_ones():
    A = wl.rmat_csr(scale=10, avg_degree=8, seed=1, values="rownorm")
    ones = np.ones((A.K, 3), np.float32)
    y = oracle.spmm_ref(A.M, A.K, 3, A.rowptr, A.colidx, A.vals, ones, with_bound=False)
    lens = A.row_lengths()
    assert np.all(y[lens == 0] == 0.0)
    assert np.allclose(y[lens > 0], 1.0, rtol=0, atol=1e-6)


# ---------------------------------------------------------------- acceptance helper and features
def test_within_bound_helper():
    yref = np.array([[1.0, 0.0]])
    bnd = np.array([[2.0, 0.0]])
    assert oracle.within_bound(np.array([[1.0 + 1e-5, 0.0]]), yref, bnd)[0]
    assert not oracle.within_bound(np.array([[1.0 + 3e-5, 0.0]]), yref, bnd)[0]
    assert not oracle.within_bound(np.array([[1.0, 1e-30]]), yref, bnd)[0]   # bound 0 => exact 0


def test_row_features_closed_forms():
    f = oracle.row_features(np.array([0, 0, 1, 3, 6]))          # lengths 0,1,2,3
    assert f["avg_row"] == 1.5 and abs(f["stdv_row"] - np.sqrt(1.25)) < 1e-15
    assert (f["max_row"], f["min_row"], f["nnz"], f["M"]) == (3, 0, 6, 4)
    f = oracle.row_features(np.arange(0, 7 * 100 + 1, 7))       # every row has 7
    assert f["avg_row"] == 7.0 and f["stdv_row"] == 0.0
    # two-point law: half the rows 2, half 10 -> mean 6, std 4
    lens = np.array([2, 10] * 50)
    f = oracle.row_features(np.concatenate(([0], np.cumsum(lens))))
    assert f["avg_row"] == 6.0 and f["stdv_row"] == 4.0
