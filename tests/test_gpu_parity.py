"""GPU parity: every kernel, through the C-ABI, against the CPU oracle.

Acceptance (elementwise, summation order differs between kernels):
    |Y - Yref| <= 1e-5 * (|A| |X|)
Entries whose bound is zero (empty rows) must be exactly 0.
"""
import numpy as np
import pytest

import oracle
from paper_2106_16064_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-5
ALGO_NAMES = {0: "rs_sr", 1: "rs_pr", 2: "nb_sr", 3: "nb_pr"}


@pytest.fixture(scope="module")
def dg():
    import torch
    from paper_2106_16064_amd import binding
    assert torch.cuda.is_available()
    binding.lib()          # fails loudly if libdgsp.so is missing
    return binding


def _device_run(dg, A, X, algo, use_nnz=True, x_offset=0, y_offset=0, poison=True):
    """Runs one kernel; X / Y may be placed `offset` floats into a larger buffer
    to exercise the narrower vector paths."""
    import torch
    dev = "cuda:0"
    K, N = X.shape
    dA = dg.DeviceCsr(A, dev)
    xbuf = torch.empty(K * N + x_offset + 4, dtype=torch.float32, device=dev)
    dX = xbuf[x_offset:x_offset + K * N]
    dX.copy_(torch.from_numpy(X.reshape(-1)))
    ybuf = torch.full((A.M * N + y_offset + 4,), float("nan") if poison else 0.0, dtype=torch.float32, device=dev)
    dY = ybuf[y_offset:y_offset + A.M * N]
    if use_nnz:
        dg.dgsp_spmm_csr_nnz(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, algo)
    else:
        dg.dgsp_spmm_csr(A.M, A.K, N, dA.rowptr, dA.colidx, dA.vals, dX, dY, algo)
    torch.cuda.synchronize()
    out = ybuf.cpu().numpy()
    # nothing outside Y may be touched
    guard = np.concatenate([out[:y_offset], out[y_offset + A.M * N:]])
    assert np.all(np.isnan(guard)) if poison else np.all(guard == 0)
    return out[y_offset:y_offset + A.M * N].reshape(A.M, N)


def check(dg, A, X, algos=(0, 1, 2, 3), use_nnz=True, x_offset=0, y_offset=0, ref=None):
    K, N = X.shape
    yref, bnd = ref if ref is not None else oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    for algo in algos:
        print(f"[case] {A.name} M={A.M} nnz={A.nnz} N={N} algo={ALGO_NAMES[algo]} nnz_hint={use_nnz} "
              f"xoff={x_offset} yoff={y_offset}", flush=True)
        Y = _device_run(dg, A, X, algo, use_nnz, x_offset, y_offset)
        assert not np.isnan(Y).any(), f"{ALGO_NAMES[algo]}: some outputs were never written"
        ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
        assert ok, f"{ALGO_NAMES[algo]} on {A.name} N={N}: worst |err|/bound = {worst:.3e}"
    return yref, bnd


# ------------------------------------------------------------------ benchmark configs, small and medium
@pytest.mark.parametrize("use_nnz", [True, False])
def test_tiny_poisson_config(dg, use_nnz):
    A = wl.poisson_csr(4096, 4096, 8.0, seed=0)
    check(dg, A, wl.dense_matrix(A.K, 4, "uniform", seed=0), use_nnz=use_nnz)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 8, 16, 17, 32, 33, 64, 100, 128, 256, 260, 512, 520])
def test_dense_widths(dg, N):
    A = wl.poisson_csr(3000, 2500, 9.0, seed=N)
    check(dg, A, wl.dense_matrix(A.K, N, "normal", seed=N))


@pytest.mark.parametrize("N", [1, 4, 32])
def test_rmat_medium(dg, N):
    A = wl.rmat_csr(scale=15, avg_degree=16, seed=2, values="uniform01" if N == 1 else "rownorm")
    check(dg, A, wl.dense_matrix(A.K, N, "normal", seed=1))
    check(dg, A, wl.dense_matrix(A.K, N, "normal", seed=1), use_nnz=False)


@pytest.mark.parametrize("N", [1, 2, 4, 8])
def test_stencil_medium(dg, N):
    A = wl.stencil27_csr(24, seed=1)
    check(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=2))


@pytest.mark.parametrize("dist", wl.SWEEP_DISTS)
@pytest.mark.parametrize("N", [1, 8, 64])
def test_sweep_laws(dg, dist, N):
    A = wl.sweep_csr(1 << 14, 16, dist, seed=0)
    check(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=3))


# ------------------------------------------------------------------ structure edge cases
def test_row_lengths_around_wave_and_tile_edges(dg):
    lens = [0, 1, 2, 63, 64, 65, 0, 0, 127, 128, 129, 255, 256, 257, 511, 512, 513, 1, 0, 1023, 1024, 1025, 3, 0]
    A = wl.csr_from_lens(lens * 7, K=5000, seed=1, name="edges")
    for N in (1, 2, 4, 8, 32, 64):
        check(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=N))


def test_single_long_row_and_long_tail(dg):
    A = wl.csr_from_lens([20000] + [1] * 300 + [0] * 50 + [7000], K=30000, seed=2, name="long_rows")
    for N in (1, 4, 16, 128):
        check(dg, A, wl.dense_matrix(A.K, N, "normal", seed=N))


def test_many_empty_rows_between_entries(dg):
    # more row starts inside one tile than the LDS window holds: the search falls back to global memory
    lens = np.zeros(200000, dtype=np.int64)
    lens[::997] = 3
    lens[123456] = 900
    A = wl.csr_from_lens(lens, K=777, seed=3, name="mostly_empty")
    for N in (1, 4, 8, 64):
        check(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=N))
        check(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=N), use_nnz=False)


def test_all_rows_empty_and_no_rows(dg):
    A = wl.csr_from_lens([0] * 1000, K=10, seed=0, name="all_empty")
    for N in (1, 4, 7, 64):
        Y = check(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=0))
        check(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=0), use_nnz=False)


def test_zero_extents_return_ok(dg):
    import torch
    e32 = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    ef = torch.zeros(0, dtype=torch.float32, device="cuda:0")
    ei = torch.zeros(0, dtype=torch.int32, device="cuda:0")
    for algo in range(4):
        dg.dgsp_spmm_csr(0, 5, 3, e32, ei, ef, torch.zeros(15, device="cuda:0"), ef, algo)
    rp = torch.zeros(6, dtype=torch.int32, device="cuda:0")
    for algo in range(4):
        dg.dgsp_spmm_csr(5, 5, 0, rp, ei, ef, ef, ef, algo)
    torch.cuda.synchronize()


def test_one_row_one_entry(dg):
    A = wl.csr_from_lens([1], K=1, seed=0, name="1x1")
    for N in (1, 2, 3, 4, 64):
        check(dg, A, wl.dense_matrix(1, N, "uniform", seed=N))


def test_tall_skinny_and_wide(dg):
    A = wl.csr_from_lens(np.full(50000, 2), K=3, seed=1, name="tall")
    check(dg, A, wl.dense_matrix(3, 8, "uniform", seed=1))
    B = wl.csr_from_lens([40000, 40000, 40000], K=50000, seed=1, name="wide")
    check(dg, B, wl.dense_matrix(50000, 2, "uniform", seed=1))


@pytest.mark.parametrize("N,xoff,yoff", [(4, 1, 0), (4, 0, 1), (4, 2, 2), (8, 3, 1), (2, 1, 1), (64, 2, 0)])
def test_buffers_at_odd_dword_addresses(dg, N, xoff, yoff):
    """X and Y a few floats into their allocations: the multi-dword accesses of every kernel then start at
    addresses that are multiples of 4 bytes only; nothing next to Y may change."""
    A = wl.poisson_csr(2000, 2000, 12.0, seed=5)
    check(dg, A, wl.dense_matrix(A.K, N, "normal", seed=5), x_offset=xoff, y_offset=yoff)


def test_unsorted_columns_and_duplicates(dg):
    rng = np.random.default_rng(0)
    A = wl.poisson_csr(3000, 500, 20.0, seed=8)
    colidx = A.colidx.copy()
    for i in range(A.M):
        s, e = A.rowptr[i], A.rowptr[i + 1]
        colidx[s:e] = rng.permutation(colidx[s:e])
    colidx[rng.integers(0, A.nnz, 2000)] = 7        # plenty of repeated (row, col) pairs
    B = wl.CsrMatrix(A.M, A.K, A.rowptr, colidx, A.vals, "unsorted_dups")
    check(dg, B, wl.dense_matrix(B.K, 4, "uniform", seed=1))
    check(dg, B, wl.dense_matrix(B.K, 32, "uniform", seed=1))


# ------------------------------------------------------------------ exact invariants
def test_identity_is_bit_exact(dg):
    K = 10000
    I = wl.CsrMatrix(K, K, np.arange(K + 1, dtype=np.int32), np.arange(K, dtype=np.int32),
                     np.ones(K, np.float32), "identity")
    for N in (1, 4, 32):
        X = wl.dense_matrix(K, N, "normal", seed=N)
        for algo in range(4):
            Y = _device_run(dg, I, X, algo)
            assert np.array_equal(Y, X), ALGO_NAMES[algo]


def test_single_entry_rows_equal_the_rounded_product(dg):
    rng = np.random.default_rng(4)
    M, K = 5000, 300
    A = wl.CsrMatrix(M, K, np.arange(M + 1, dtype=np.int32), rng.integers(0, K, M).astype(np.int32),
                     rng.uniform(-1, 1, M).astype(np.float32), "one_per_row")
    X = wl.dense_matrix(K, 4, "uniform", seed=4)
    want = A.vals[:, None] * X[A.colidx]            # one fp32 rounding
    for algo in range(4):
        assert np.array_equal(_device_run(dg, A, X, algo), want), ALGO_NAMES[algo]


def test_balanced_kernels_agree_with_themselves(dg):
    # atomics make the balanced kernels order-dependent, but only within rounding
    A = wl.rmat_csr(scale=14, avg_degree=16, seed=3)
    X = wl.dense_matrix(A.K, 4, "uniform", seed=0)
    yref, bnd = oracle.spmm_ref(A.M, A.K, 4, A.rowptr, A.colidx, A.vals, X)
    for algo in (2, 3):
        y1 = _device_run(dg, A, X, algo)
        y2 = _device_run(dg, A, X, algo)
        assert np.all(np.abs(y1.astype(np.float64) - y2) <= 2 * TOL * bnd)


# ------------------------------------------------------------------ adaptive entry point and helpers
def test_auto_entry_point_runs_the_selected_kernel(dg):
    import torch
    for A, N in ((wl.sweep_csr(1 << 14, 64, "fixed", 0), 1), (wl.sweep_csr(1 << 14, 4, "zipf", 0), 2),
                 (wl.sweep_csr(1 << 14, 16, "poisson", 0), 64), (wl.sweep_csr(1 << 14, 64, "zipf", 0), 64)):
        X = wl.dense_matrix(A.K, N, "uniform", seed=1)
        dA = dg.DeviceCsr(A)
        dX = torch.from_numpy(X).cuda()
        dY = torch.full((A.M, N), float("nan"), device="cuda:0")
        chosen = dg.dgsp_spmm_csr_auto(A.M, A.K, N, dA.features, dA.rowptr, dA.colidx, dA.vals, dX, dY)
        assert chosen == dg.dgsp_select_algo(dA.features, N) and chosen in range(4)
        yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
        ok, worst = oracle.within_bound(dY.cpu().numpy(), yref, bnd, TOL)
        assert ok, (A.name, N, chosen, worst)
        # AUTO without features falls back to the balanced kernels
        dY.fill_(float("nan"))
        dg.dgsp_spmm_csr(A.M, A.K, N, dA.rowptr, dA.colidx, dA.vals, dX, dY, dg.AUTO)
        assert oracle.within_bound(dY.cpu().numpy(), yref, bnd, TOL)[0]


def test_works_on_a_side_stream(dg):
    import torch
    A = wl.poisson_csr(20000, 20000, 10.0, seed=9)
    X = wl.dense_matrix(A.K, 8, "uniform", seed=9)
    yref, bnd = oracle.spmm_ref(A.M, A.K, 8, A.rowptr, A.colidx, A.vals, X)
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).cuda()
    s = torch.cuda.Stream()
    for algo in range(4):
        dY = torch.full((A.M, 8), float("nan"), device="cuda:0")
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            dg.dgsp_spmm_csr_nnz(A.M, A.K, 8, A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, algo)
        s.synchronize()
        assert oracle.within_bound(dY.cpu().numpy(), yref, bnd, TOL)[0]


def test_invalid_arguments_are_rejected(dg):
    import torch
    A = wl.poisson_csr(100, 100, 4.0, seed=0)
    dA = dg.DeviceCsr(A)
    X = torch.zeros(100, 2, device="cuda:0")
    Y = torch.zeros(100, 2, device="cuda:0")
    L = dg.lib()
    args = lambda algo, M=100, N=2: (M, 100, N, dA.rowptr.data_ptr(), dA.colidx.data_ptr(), dA.vals.data_ptr(),
                                     X.data_ptr(), Y.data_ptr(), algo, None)
    assert L.dgsp_spmm_csr(*args(7)) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr(*args(-2)) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr(*args(0, M=-1)) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr(100, 100, 2, None, None, None, None, None, 0, None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr(*args(0)) == dg.OK
    torch.cuda.synchronize()


def test_copy_kernel(dg):
    import torch
    for n in (0, 1, 5, 4096, 1000003):
        src = torch.randn(n + 8, device="cuda:0")[:n] if n else torch.zeros(0, device="cuda:0")
        base = torch.zeros(n + 4, device="cuda:0")
        dg.dgsp_copy_f32(base[:n], src, n)
        torch.cuda.synchronize()
        assert torch.equal(base[:n], src) and torch.all(base[n:] == 0)


def test_phase_entry_point_equals_the_whole_call(dg):
    import torch
    A = wl.rmat_csr(scale=13, avg_degree=16, seed=5)
    X = wl.dense_matrix(A.K, 4, "uniform", seed=2)
    yref, bnd = oracle.spmm_ref(A.M, A.K, 4, A.rowptr, A.colidx, A.vals, X)
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).cuda()
    for algo in range(4):
        dY = torch.full((A.M, 4), float("nan"), device="cuda:0")
        dg.dgsp_spmm_csr_phase(A.M, A.K, 4, A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, algo, dg.PHASE_PREPARE)
        dg.dgsp_spmm_csr_phase(A.M, A.K, 4, A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, algo, dg.PHASE_MAIN)
        torch.cuda.synchronize()
        ok, worst = oracle.within_bound(dY.cpu().numpy(), yref, bnd, TOL)
        assert ok, (ALGO_NAMES[algo], worst)
    L = dg.lib()
    assert L.dgsp_spmm_csr_phase(A.M, A.K, 4, A.nnz, dA.rowptr.data_ptr(), dA.colidx.data_ptr(), dA.vals.data_ptr(),
                                 dX.data_ptr(), dY.data_ptr(), -1, 0, None, None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr_phase(A.M, A.K, 4, A.nnz, dA.rowptr.data_ptr(), dA.colidx.data_ptr(), dA.vals.data_ptr(),
                                 dX.data_ptr(), dY.data_ptr(), 0, 5, None, None) == dg.ERR_INVALID_ARG


def test_gather_probe_sums_every_gathered_value(dg):
    import torch
    n, K = 1000003, 5000
    idx = torch.randint(0, K, (n,), dtype=torch.int32, device="cuda:0")
    x = torch.randint(-4, 5, (K,), device="cuda:0").float()          # small integers: sums are exact
    out = torch.empty(dg.dgsp_gather_probe_out_len(), device="cuda:0")
    dg.dgsp_gather_probe(out, x, idx)
    torch.cuda.synchronize()
    assert out.double().sum().item() == x[idx.long()].double().sum().item()


@pytest.mark.parametrize("mode,N", [(0, 1), (1, 1), (1, 2), (1, 4), (2, 8), (2, 32), (2, 64), (2, 128), (2, 36)])
def test_floor_probes_touch_every_entry_once(dg, mode, N):
    """The floor probes (memory side of the kernels, no rows) are measurement aids, but what they read is checked:
    their partial sums add up to the sum of all elements of A X, which the oracle gives.  Small integer values keep
    every fp32 partial sum exact, so the comparison is equality."""
    import torch
    A = wl.rmat_csr(scale=13, avg_degree=12, seed=21)
    rng = np.random.default_rng(22)
    vals = rng.integers(-2, 3, size=A.nnz).astype(np.float32)
    if mode == 0:
        vals[:] = 1.0                                        # the bare gather does not read the values
    X = rng.integers(-3, 4, size=(A.K, N)).astype(np.float32)
    yref, _ = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, vals, X)
    n_out = dg.dgsp_floor_probe_out_len(mode, N)
    assert n_out > 0
    out = torch.full((n_out,), float("nan"), device="cuda:0")
    dg.dgsp_floor_probe(mode, A.K, N, torch.from_numpy(A.colidx).cuda(), torch.from_numpy(vals).cuda(),
                        torch.from_numpy(X).cuda(), out)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(out).any())
    assert out.double().sum().item() == yref.sum()


def test_floor_probe_rejects_what_it_does_not_offer(dg):
    import torch
    L = dg.lib()
    assert dg.dgsp_floor_probe_out_len(1, 3) == -1 and dg.dgsp_floor_probe_out_len(2, 6) == -1
    assert dg.dgsp_floor_probe_out_len(7, 1) == -1
    buf = torch.zeros(16, device="cuda:0")
    idx = torch.zeros(16, dtype=torch.int32, device="cuda:0")
    args = (idx.data_ptr(), buf.data_ptr(), buf.data_ptr(), buf.data_ptr(), None)
    assert L.dgsp_floor_probe(1, 16, 4, 3, *args) == dg.ERR_UNSUPPORTED
    assert L.dgsp_floor_probe(2, 16, 4, 6, *args) == dg.ERR_UNSUPPORTED
    assert L.dgsp_floor_probe(0, 16, 4, 2, *args) == dg.ERR_UNSUPPORTED
    assert L.dgsp_floor_probe(9, 16, 4, 1, *args) == dg.ERR_INVALID_ARG
    assert L.dgsp_floor_probe(1, -1, 4, 1, *args) == dg.ERR_INVALID_ARG
    assert L.dgsp_floor_probe(1, 16, 4, 1, idx.data_ptr(), buf.data_ptr(), buf.data_ptr(), None, None) == dg.ERR_INVALID_ARG


@pytest.mark.parametrize("N", [1, 2, 6, 8, 64])
def test_column_span_hint_changes_nothing_but_speed(dg, N):
    """With a matrix's features (banded: small col_span) the sequential kernels keep more loads in flight."""
    import torch
    A = wl.stencil27_csr(48, seed=3)
    X = wl.dense_matrix(A.K, N, "uniform", seed=N)
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    dA = dg.DeviceCsr(A)
    assert 0 < dA.features.col_span <= 0.05
    dX = torch.from_numpy(X).cuda()
    for algo in range(4):
        dY = torch.full((A.M, N), float("nan"), device="cuda:0")
        dA.spmm(dX, algo=algo, Y=dY)          # passes the features along with the named kernel
        torch.cuda.synchronize()
        ok, worst = oracle.within_bound(dY.cpu().numpy(), yref, bnd, TOL)
        assert ok, (ALGO_NAMES[algo], N, worst)


# ------------------------------------------------------------------ optimisations switched off (Sections 2.1.2, 2.1.3)
def _ablation_run(dg, A, X, algo, switches):
    import torch
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).to("cuda:0")
    dY = torch.full((A.M, X.shape[1]), float("nan"), dtype=torch.float32, device="cuda:0")
    dg.dgsp_spmm_csr_ablation(A.M, A.K, X.shape[1], A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, algo, switches,
                              dA.features)
    torch.cuda.synchronize()
    return dY.cpu().numpy()


@pytest.mark.parametrize("N", [1, 2, 4, 7, 8, 64, 130])
def test_switched_off_optimisations_compute_the_same_product(dg, N):
    """Scalar dense-row loads (all four kernels) and the sequential kernel without its LDS tile
    change the schedule only: same acceptance bound against the oracle."""
    A = wl.sweep_csr(3000, 16, "lognormal", seed=N)
    X = wl.dense_matrix(A.K, N, "normal", seed=N)
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    cases = [(a, dg.ABL_SCALAR_DENSE_LOADS) for a in (0, 1, 2, 3)]
    cases += [(0, dg.ABL_NO_SPARSE_STAGING), (0, dg.ABL_NO_SPARSE_STAGING | dg.ABL_SCALAR_DENSE_LOADS), (3, 0)]
    cases += [(3, dg.ABL_ITEM_TILES), (3, dg.ABL_ITEM_TILES | dg.ABL_SCALAR_DENSE_LOADS)]
    cases += [(3, dg.ABL_SERIAL_SEGMENT_SCAN | dg.ABL_SCALAR_DENSE_LOADS)] + ([(3, dg.ABL_SERIAL_SEGMENT_SCAN)] if N in (1, 2, 130) else [])
    for algo, sw in cases:
        print(f"[case] ablation N={N} algo={ALGO_NAMES[algo]} switches={sw}", flush=True)
        Y = _ablation_run(dg, A, X, algo, sw)
        assert not np.isnan(Y).any()
        ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
        assert ok, f"{ALGO_NAMES[algo]} switches={sw} N={N}: worst |err|/bound = {worst:.3e}"


@pytest.mark.parametrize("N", [1, 2, 3, 4, 9, 12])
@pytest.mark.parametrize("kind", ["rmat", "mostly_empty", "hub", "stencil"])
def test_both_pipelines_of_the_balanced_parallel_kernel(dg, kind, N):
    """At up to four dense columns per lane DGSP_NB_PR can walk blocks of entries (gathers requested a block ahead)
    or tiles of merge-path items; the ablation switches force one or the other at any size.  Both against the
    oracle, on structures that stress what differs: long stretches of empty rows (several steps per block), rows
    spanning many blocks, and short regular rows; N = 9 and 12 run several passes of three and four columns.  The
    third variant (one or two columns per lane only) replaces the DPP segment reduction by a serial scan (the
    comparison kernel of Section 2.1.1)."""
    if kind == "rmat":
        A = wl.rmat_csr(scale=15, avg_degree=16, seed=31)
    elif kind == "mostly_empty":
        lens = np.zeros(300000, dtype=np.int64); lens[::1013] = 3; lens[150000] = 5000
        A = wl.csr_from_lens(lens, 8192, seed=32, name="mostly_empty")
    elif kind == "hub":
        lens = np.full(5000, 1); lens[17] = 30000; lens[4000] = 9000; lens[100:900] = 0
        A = wl.csr_from_lens(lens, 40000, seed=33, name="hub")
    else:
        A = wl.stencil27_csr(24, seed=34)
    X = wl.dense_matrix(A.K, N, "uniform", seed=35 + N)
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    for sw in (0, dg.ABL_ITEM_TILES, dg.ABL_ENTRY_BLOCKS) + ((dg.ABL_SERIAL_SEGMENT_SCAN,) if N <= 2 else ()):
        print(f"[case] nb_pr pipelines {kind} N={N} switches={sw}", flush=True)
        Y = _ablation_run(dg, A, X, dg.NB_PR, sw)
        assert not np.isnan(Y).any()
        ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
        assert ok, f"{kind} N={N} switches={sw}: worst |err|/bound = {worst:.3e}"
        assert np.all(Y[A.row_lengths() == 0] == 0.0)


@pytest.mark.parametrize("N", [32, 64, 128, 256])
def test_wide_column_layouts_of_the_balanced_sequential_kernel(dg, N):
    """Column blocks of 32 instead of 64 dense columns, and column blocks as a grid dimension instead of tied to
    XCDs: comparison layouts of DGSP_NB_SR for wide X, same product (the shipped layout is what every other test of
    the kernel at N >= 128 runs)."""
    A = wl.rmat_csr(scale=14, avg_degree=16, seed=41)
    X = wl.dense_matrix(A.K, N, "normal", seed=42)
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    for sw in (dg.ABL_COLUMN_BLOCKS_32, dg.ABL_BLOCKS_OFF_XCDS, dg.ABL_COLUMN_BLOCKS_32 | dg.ABL_BLOCKS_OFF_XCDS):
        print(f"[case] nb_sr layouts N={N} switches={sw}", flush=True)
        Y = _ablation_run(dg, A, X, dg.NB_SR, sw)
        assert not np.isnan(Y).any()
        ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
        assert ok, f"N={N} switches={sw}: worst |err|/bound = {worst:.3e}"
        assert np.all(Y[A.row_lengths() == 0] == 0.0)


def test_ablation_entry_rejects_what_it_does_not_offer(dg):
    import torch
    A = wl.poisson_csr(64, 64, 4.0, seed=0)
    dA = dg.DeviceCsr(A)
    X = torch.zeros((A.K, 2), device="cuda:0")
    Y = torch.zeros((A.M, 2), device="cuda:0")
    L = dg.lib()
    args = (A.M, A.K, 2, A.nnz, dA.rowptr.data_ptr(), dA.colidx.data_ptr(), dA.vals.data_ptr(), X.data_ptr(), Y.data_ptr())
    # the same with N = 8 and N = 4 (refused before anything is launched, so the narrower X and Y do not matter)
    args8 = (A.M, A.K, 8, A.nnz, dA.rowptr.data_ptr(), dA.colidx.data_ptr(), dA.vals.data_ptr(), X.data_ptr(), Y.data_ptr())
    args4 = (A.M, A.K, 4, A.nnz, dA.rowptr.data_ptr(), dA.colidx.data_ptr(), dA.vals.data_ptr(), X.data_ptr(), Y.data_ptr())
    assert L.dgsp_spmm_csr_ablation(*args, dg.NB_SR, dg.ABL_NO_SPARSE_STAGING, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args, dg.RS_SR, 1 << 12, None, None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr_ablation(*args, dg.NB_SR, dg.ABL_ITEM_TILES, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args, dg.RS_PR, dg.ABL_SERIAL_SEGMENT_SCAN, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args, dg.NB_PR, dg.ABL_COLUMN_BLOCKS_32, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args, dg.NB_PR, dg.ABL_ENTRY_BLOCKS | dg.ABL_ITEM_TILES, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args8, dg.NB_PR, dg.ABL_ENTRY_BLOCKS, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args, dg.NB_SR, dg.ABL_ENTRY_BLOCKS, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args, dg.RS_SR, dg.ABL_BLOCKS_OFF_XCDS, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args, dg.NB_PR, dg.ABL_SERIAL_SEGMENT_SCAN | dg.ABL_ITEM_TILES, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args4, dg.NB_PR, dg.ABL_SERIAL_SEGMENT_SCAN, None, None) == dg.ERR_UNSUPPORTED
    assert L.dgsp_spmm_csr_ablation(*args, dg.AUTO, 0, None, None) == dg.ERR_INVALID_ARG
    torch.cuda.synchronize()


# ------------------------------------------------------------------ row statistics on the device, profile-based selection
@pytest.mark.parametrize("gen", ["poisson", "rmat", "stencil", "hub", "unsorted", "empty_rows"])
def test_device_features_equal_the_host_ones(dg, gen):
    """Section 2.2's metrics computed by the GPU from device CSR: integer sums, so bit-equal to the
    host pass, which tests/test_host_api.py pins to closed forms and to the oracle's statistics."""
    import torch
    if gen == "poisson":
        A = wl.poisson_csr(5000, 3000, 6.0, seed=1)
    elif gen == "rmat":
        A = wl.rmat_csr(scale=14, avg_degree=16, seed=3)
    elif gen == "stencil":
        A = wl.stencil27_csr(17, seed=0)
    elif gen == "hub":
        lens = np.full(3000, 2); lens[7] = 2900; lens[2999] = 700; lens[100:200] = 0
        A = wl.csr_from_lens(lens, 3000, seed=5, name="hub")
    elif gen == "unsorted":
        A = wl.sweep_csr(2000, 16, "lognormal", seed=2)
        rng = np.random.default_rng(0)
        for i in range(A.M):           # shuffle the columns inside every row
            s, e = A.rowptr[i], A.rowptr[i + 1]
            A.colidx[s:e] = rng.permutation(A.colidx[s:e])
    else:
        lens = np.zeros(1000, dtype=np.int64); lens[::97] = 5
        A = wl.csr_from_lens(lens, 1 << 20, seed=6, name="mostly_empty")
    host = dg.dgsp_features_from_csr_host(A.M, A.K, A.rowptr, A.colidx)
    rp = torch.from_numpy(A.rowptr).cuda()
    ci = torch.from_numpy(A.colidx).cuda()
    dev = dg.dgsp_features_from_csr_device(A.M, A.K, rp, ci)
    for name in ("M", "K", "nnz", "max_row", "min_row", "avg_row", "stdv_row", "cv_row", "col_span"):
        assert getattr(dev, name) == getattr(host, name), name
    # and against the oracle's own statistics (numpy)
    ref = oracle.row_features(A.rowptr)
    assert (dev.nnz, dev.max_row, dev.min_row) == (ref["nnz"], ref["max_row"], ref["min_row"])
    assert dev.avg_row == pytest.approx(ref["avg_row"], rel=1e-12)
    assert dev.stdv_row == pytest.approx(ref["stdv_row"], rel=1e-9, abs=1e-12)
    # col_span against its definition, written out with numpy on the host copy
    lens = np.diff(A.rowptr)
    spans = [int(A.colidx[s:e].max()) - int(A.colidx[s:e].min()) + 1
             for s, e in zip(A.rowptr[:-1], A.rowptr[1:]) if e > s]
    assert dev.col_span == pytest.approx(sum(spans) / (A.K * len(spans)) if spans else 0.0, rel=1e-12)
    assert int((lens > 0).sum()) == len(spans)
    # without colidx the row statistics are the same and col_span stays 0
    dev2 = dg.dgsp_features_from_csr_device(A.M, A.K, rp, None)
    assert dev2.col_span == 0.0 and dev2.stdv_row == host.stdv_row and dev2.nnz == host.nnz


def test_device_features_reject_malformed_input(dg):
    import torch
    L = dg.lib()
    f = dg.Features()
    ws = torch.empty(8, dtype=torch.int64, device="cuda:0")
    bad = torch.tensor([0, 3, 2, 5], dtype=torch.int32, device="cuda:0")        # decreases
    assert L.dgsp_features_from_csr_device(3, 8, bad.data_ptr(), None, ws.data_ptr(), ctypes_byref(f), None) == dg.ERR_INVALID_ARG
    off = torch.tensor([1, 3, 4, 5], dtype=torch.int32, device="cuda:0")        # does not start at 0
    assert L.dgsp_features_from_csr_device(3, 8, off.data_ptr(), None, ws.data_ptr(), ctypes_byref(f), None) == dg.ERR_INVALID_ARG
    ok = torch.tensor([0, 3, 4, 5], dtype=torch.int32, device="cuda:0")
    assert L.dgsp_features_from_csr_device(3, 8, ok.data_ptr(), None, None, ctypes_byref(f), None) == dg.ERR_INVALID_ARG
    assert L.dgsp_features_from_csr_device(3, 8, ok.data_ptr(), None, ws.data_ptr() + 4, ctypes_byref(f), None) == dg.ERR_INVALID_ARG
    assert L.dgsp_features_from_csr_device(0, 8, None, None, None, ctypes_byref(f), None) == dg.OK and f.nnz == 0
    assert L.dgsp_features_from_csr_device(3, 8, ok.data_ptr(), None, ws.data_ptr(), ctypes_byref(f), None) == dg.OK
    assert (f.nnz, f.max_row, f.min_row) == (5, 3, 1)


def ctypes_byref(x):
    import ctypes
    return ctypes.byref(x)


@pytest.mark.parametrize("N", [1, 8])
def test_autotune_reports_the_fastest_kernel_and_leaves_the_product(dg, N):
    import torch
    A = wl.rmat_csr(scale=15, avg_degree=16, seed=4)
    X = wl.dense_matrix(A.K, N, "uniform", seed=4)
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).cuda()
    dY = torch.full((A.M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    best, ms = dg.dgsp_autotune(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, dA.features, reps=3)
    assert best in (0, 1, 2, 3) and len(ms) == 4
    assert all(np.isfinite(t) and t > 0 for t in ms)
    assert ms[best] == min(ms)
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    ok, worst = oracle.within_bound(dY.cpu().numpy(), yref, bnd, TOL)
    assert ok, worst
    # a skewed graph: the row-split sequential kernel cannot be the winner
    assert best != dg.RS_SR
    # the matrix object remembers the winner and uses it for AUTO calls of that width
    b2, _ = dA.autotune(dX, reps=2)
    assert dA.tuned[N] == b2
    Y2 = dA.spmm(dX)
    ok, worst = oracle.within_bound(Y2.cpu().numpy(), yref, bnd, TOL)
    assert ok, worst


def test_forty_million_rows_mostly_empty(dg):
    """Row counts far beyond the entry count: the merge-path positions row + rowptr[row] approach
    2^26 while almost every item is a row-end marker (exercises the partition arithmetic, the
    64-row output batches and the prepare launch at a size no other test reaches)."""
    M, K = 40_000_000, 1000
    rng = np.random.default_rng(11)
    lens = np.zeros(M, dtype=np.int64)
    hot = rng.choice(M, size=200_000, replace=False)
    lens[hot] = rng.integers(1, 9, size=hot.size)
    lens[12_345_678] = 5000                       # one long row in the middle of nowhere
    A = wl.csr_from_lens(np.minimum(lens, K), K, seed=12, name="forty_million_rows")
    X = wl.dense_matrix(K, 1, "uniform", seed=3)
    ref = oracle.spmm_ref(A.M, A.K, 1, A.rowptr, A.colidx, A.vals, X)
    check(dg, A, X, algos=(0, 1, 2, 3), ref=ref)


# ------------------------------------------------------------------ strided views (leading dimensions)
@pytest.mark.parametrize("N,ldx,ldy,x0,y0", [
    (1, 8, 4, 0, 0), (1, 7, 3, 5, 2), (2, 8, 8, 2, 4), (2, 9, 5, 1, 3), (4, 16, 8, 4, 4), (4, 12, 12, 3, 0),
    (8, 128, 64, 32, 8), (32, 128, 128, 64, 96), (33, 70, 40, 1, 7), (100, 260, 104, 4, 0), (64, 64, 64, 0, 0),
])
def test_column_slices_of_wider_matrices(dg, N, ldx, ldy, x0, y0):
    """Y[:, y0:y0+N] = A X[:, x0:x0+N] on views of row-major matrices with ldx / ldy floats per row:
    the product equals the oracle's on the packed copy, and nothing outside the slice is written."""
    import torch
    A = wl.sweep_csr(2500, 12, "lognormal", seed=N + ldx)
    rng = np.random.default_rng(N * 1000 + ldx)
    Xw = rng.standard_normal((A.K, ldx)).astype(np.float32)
    Xs = np.ascontiguousarray(Xw[:, x0:x0 + N])
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, Xs)
    dA = dg.DeviceCsr(A)
    dXw = torch.from_numpy(Xw).cuda()
    for algo in (0, 1, 2, 3, dg.AUTO):
        print(f"[case] strided N={N} ldx={ldx} ldy={ldy} x0={x0} y0={y0} algo={algo}", flush=True)
        dYw = torch.full((A.M, ldy), float("nan"), dtype=torch.float32, device="cuda:0")
        dg.dgsp_spmm_csr_ld(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, dXw[:, x0:x0 + N],
                            dYw[:, y0:y0 + N], algo, dA.features)
        torch.cuda.synchronize()
        Yw = dYw.cpu().numpy()
        Y = Yw[:, y0:y0 + N]
        assert not np.isnan(Y).any()
        ok, worst = oracle.within_bound(Y, yref, bnd, TOL)
        assert ok, f"algo {algo}: worst |err|/bound = {worst:.3e}"
        outside = np.ones(ldy, dtype=bool); outside[y0:y0 + N] = False
        assert np.isnan(Yw[:, outside]).all(), "wrote outside the slice"


def test_leading_dimensions_smaller_than_the_width_are_rejected(dg):
    import torch
    A = wl.poisson_csr(64, 64, 4.0, seed=0)
    dA = dg.DeviceCsr(A)
    X = torch.zeros((A.K, 8), device="cuda:0")
    Y = torch.zeros((A.M, 8), device="cuda:0")
    L = dg.lib()
    base = (A.M, A.K, 8, A.nnz, dA.rowptr.data_ptr(), dA.colidx.data_ptr(), dA.vals.data_ptr())
    assert L.dgsp_spmm_csr_ld(*base, X.data_ptr(), 7, Y.data_ptr(), 8, dg.NB_SR, None, None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr_ld(*base, X.data_ptr(), 8, Y.data_ptr(), 4, dg.NB_SR, None, None) == dg.ERR_INVALID_ARG
    assert L.dgsp_spmm_csr_ld(*base, X.data_ptr(), 8, Y.data_ptr(), 8, dg.NB_SR, None, None) == dg.OK
    torch.cuda.synchronize()


# ------------------------------------------------------------------ HIP graph capture
@pytest.mark.parametrize("algo", [0, 1, 2, 3])
def test_calls_can_be_captured_in_a_graph_and_replayed(dg, algo):
    """The library allocates nothing and only launches kernels, so a call can be recorded into a HIP
    graph.  Every replay is checked against the oracle, with eager work and new inputs in between."""
    import torch
    A = wl.poisson_csr(4096, 4096, 8.0, seed=3)
    N = 4
    dA = dg.DeviceCsr(A)
    dX = torch.zeros((A.K, N), dtype=torch.float32, device="cuda:0")
    dY = torch.zeros((A.M, N), dtype=torch.float32, device="cuda:0")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):                     # one eager call first: fills the library's host-side caches
        dA.spmm(dX, algo=algo, Y=dY)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        dA.spmm(dX, algo=algo, Y=dY)                  # recorded on the capturing stream
    for rep in range(3):
        X = wl.dense_matrix(A.K, N, "uniform", seed=100 + rep)
        dX.copy_(torch.from_numpy(X))
        dY.fill_(float("nan"))                        # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
        ok, worst = oracle.within_bound(dY.cpu().numpy(), yref, bnd, TOL)
        assert ok, f"replay {rep}: worst |err|/bound = {worst:.3e}"


# ------------------------------------------------------------------ differentiable wrapper
@pytest.mark.parametrize("N", [1, 4, 32])
def test_gradient_with_respect_to_the_dense_operand(dg, N):
    """Y = A X as an autograd operation: the forward product and dL/dX = A^T dL/dY both equal the
    oracle's products (the second on the transposed arrays) within the same bound."""
    import torch
    from paper_2106_16064_amd.autograd import SparseOperator, transpose_csr
    A = wl.rmat_csr(scale=13, avg_degree=12, seed=9)
    op = SparseOperator(A)
    X = wl.dense_matrix(A.K, N, "normal", seed=1)
    Gy = wl.dense_matrix(A.M, N, "uniform", seed=2)
    dX = torch.from_numpy(X).cuda().requires_grad_(True)
    Y = op(dX)
    Y.backward(torch.from_numpy(Gy).cuda())
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    ok, worst = oracle.within_bound(Y.detach().cpu().numpy(), yref, bnd, TOL)
    assert ok, worst
    T = transpose_csr(A)
    gref, gbnd = oracle.spmm_ref(T.M, T.K, N, T.rowptr, T.colidx, T.vals, Gy)
    ok, worst = oracle.within_bound(dX.grad.cpu().numpy(), gref, gbnd, TOL)
    assert ok, worst
    # a vector operand (SpMV) goes through the same path
    if N == 1:
        v = torch.from_numpy(X[:, 0].copy()).cuda().requires_grad_(True)
        y = op(v)
        y.sum().backward()
        gref1, gbnd1 = oracle.spmm_ref(T.M, T.K, 1, T.rowptr, T.colidx, T.vals, np.ones((A.M, 1), dtype=np.float32))
        ok, worst = oracle.within_bound(v.grad.cpu().numpy().reshape(-1, 1), gref1, gbnd1, TOL)
        assert ok, worst


def test_concurrent_calls_from_several_host_threads_and_streams(dg):
    """The library keeps no per-call state: four host threads, each with its own stream, matrix and
    kernel, run at the same time (ctypes releases the interpreter lock during a call) and every
    result equals the oracle's."""
    import threading
    import torch
    jobs = []
    for i, (algo, N) in enumerate([(0, 8), (1, 2), (2, 32), (3, 1)]):
        A = wl.sweep_csr(6000 + 500 * i, 16, "lognormal", seed=20 + i)
        X = wl.dense_matrix(A.K, N, "uniform", seed=30 + i)
        jobs.append(dict(A=A, X=X, algo=algo, dA=dg.DeviceCsr(A), dX=torch.from_numpy(X).cuda(),
                         dY=torch.full((A.M, N), float("nan"), device="cuda:0"), stream=torch.cuda.Stream(), err=None))
    torch.cuda.synchronize()

    def work(job):
        try:
            for _ in range(20):
                job["dA"].spmm(job["dX"], algo=job["algo"], Y=job["dY"], stream=job["stream"])
            job["stream"].synchronize()
        except Exception as e:          # surfaced in the main thread below
            job["err"] = e

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for j in jobs:
        assert j["err"] is None, j["err"]
        A, X = j["A"], j["X"]
        yref, bnd = oracle.spmm_ref(A.M, A.K, X.shape[1], A.rowptr, A.colidx, A.vals, X)
        ok, worst = oracle.within_bound(j["dY"].cpu().numpy(), yref, bnd, TOL)
        assert ok, f"algo {j['algo']}: worst |err|/bound = {worst:.3e}"


# ------------------------------------------------------------------ more shapes at the edges
@pytest.mark.parametrize("N", [1000, 1024, 4096])
def test_very_wide_dense_operands(dg, N):
    """Widths far beyond a wave's 64 x 4 columns: several column blocks per row (grid.y)."""
    A = wl.sweep_csr(300, 6, "lognormal", seed=N)
    check(dg, A, wl.dense_matrix(A.K, N, "uniform", seed=1))


def test_single_column_matrix_and_single_row_matrix(dg):
    """K = 1 (every entry gathers the same row of X) and M = 1 (one row holds everything)."""
    rng = np.random.default_rng(3)
    lens = rng.integers(0, 2, size=5000)
    A = wl.CsrMatrix(5000, 1, np.concatenate([[0], np.cumsum(lens)]).astype(np.int32),
                     np.zeros(int(lens.sum()), dtype=np.int32), rng.standard_normal(int(lens.sum())).astype(np.float32),
                     "one_column", {})
    for N in (1, 4, 33):
        check(dg, A, wl.dense_matrix(1, N, "normal", seed=N))
    cols = np.sort(rng.choice(20000, size=7000, replace=False)).astype(np.int32)
    B = wl.CsrMatrix(1, 20000, np.array([0, 7000], dtype=np.int32), cols,
                     rng.standard_normal(7000).astype(np.float32), "one_row", {})
    for N in (1, 2, 8, 64):
        check(dg, B, wl.dense_matrix(20000, N, "uniform", seed=N))


def test_rows_in_views_far_apart(dg):
    """A leading dimension much larger than the width: rows of X and Y 4096 floats apart."""
    import torch
    A = wl.poisson_csr(700, 600, 7.0, seed=8)
    N, ld = 8, 4096
    rng = np.random.default_rng(9)
    Xw = rng.standard_normal((A.K, ld)).astype(np.float32)
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, np.ascontiguousarray(Xw[:, 100:100 + N]))
    dA = dg.DeviceCsr(A)
    dXw = torch.from_numpy(Xw).cuda()
    for algo in (0, 1, 2, 3):
        dYw = torch.full((A.M, ld), float("nan"), dtype=torch.float32, device="cuda:0")
        dg.dgsp_spmm_csr_ld(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, dXw[:, 100:100 + N], dYw[:, 2000:2000 + N],
                            algo, dA.features)
        torch.cuda.synchronize()
        Yw = dYw.cpu().numpy()
        ok, worst = oracle.within_bound(Yw[:, 2000:2000 + N], yref, bnd, TOL)
        assert ok, (algo, worst)
        assert np.isnan(Yw[:, :2000]).all() and np.isnan(Yw[:, 2000 + N:]).all()


# ------------------------------------------------------------------ the scaled form
@pytest.mark.parametrize("N", [1, 2, 4, 8, 32, 100])
@pytest.mark.parametrize("alpha,beta", [(1.0, 0.0), (2.5, 0.0), (1.0, 1.0), (-0.75, 0.5), (0.0, 2.0)])
def test_scaled_form_alpha_beta(dg, N, alpha, beta):
    """Y = alpha * A X + beta * Y0 through every kernel: compared with alpha * Yref + beta * Y0 formed in
    fp64 from the oracle's product, bound alpha*|A||X| + |beta Y0|.  With beta = 0, Y0 is NaN on purpose."""
    import torch
    A = wl.rmat_csr(scale=13, avg_degree=10, seed=40 + N)          # hubs, many empty rows
    X = wl.dense_matrix(A.K, N, "normal", seed=N)
    Y0 = wl.dense_matrix(A.M, N, "uniform", seed=100 + N)
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    want = alpha * yref + (beta * Y0.astype(np.float64) if beta != 0.0 else 0.0)
    bound = abs(alpha) * bnd + abs(beta) * np.abs(Y0.astype(np.float64))
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).cuda()
    for algo in (0, 1, 2, 3, dg.AUTO):
        print(f"[case] axpby N={N} alpha={alpha} beta={beta} algo={algo}", flush=True)
        dY = torch.from_numpy(Y0).cuda() if beta != 0.0 else torch.full((A.M, N), float("nan"), device="cuda:0")
        dg.dgsp_spmm_csr_axpby(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, alpha, beta, algo, dA.features)
        torch.cuda.synchronize()
        Y = dY.cpu().numpy()
        assert not np.isnan(Y).any()
        ok, worst = oracle.within_bound(Y, want, bound, TOL)
        assert ok, f"algo {algo}: worst |err|/bound = {worst:.3e}"


def test_scaled_form_on_views_and_without_entries(dg):
    import torch
    A = wl.sweep_csr(1500, 9, "lognormal", seed=4)
    N, ldx, ldy = 4, 12, 8
    rng = np.random.default_rng(2)
    Xw = rng.standard_normal((A.K, ldx)).astype(np.float32)
    Yw0 = rng.standard_normal((A.M, ldy)).astype(np.float32)
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, np.ascontiguousarray(Xw[:, 4:8]))
    want = 3.0 * yref - 1.0 * Yw0[:, 4:8].astype(np.float64)
    bound = 3.0 * bnd + np.abs(Yw0[:, 4:8].astype(np.float64))
    dA = dg.DeviceCsr(A)
    dXw = torch.from_numpy(Xw).cuda()
    for algo in (0, 1, 2, 3):
        dYw = torch.from_numpy(Yw0).cuda()
        dg.dgsp_spmm_csr_axpby(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, dXw[:, 4:8], dYw[:, 4:8], 3.0, -1.0, algo,
                               dA.features)
        torch.cuda.synchronize()
        Yw = dYw.cpu().numpy()
        ok, worst = oracle.within_bound(Yw[:, 4:8], want, bound, TOL)
        assert ok, (algo, worst)
        assert np.array_equal(Yw[:, :4], Yw0[:, :4])                # the rest of Y's rows is untouched
    # a matrix without entries: Y = beta * Y
    E = wl.csr_from_lens(np.zeros(300, dtype=np.int64), 50, seed=0, name="empty")
    dE = dg.DeviceCsr(E)
    for algo in (0, 1, 2, 3):
        Y0 = rng.standard_normal((300, 2)).astype(np.float32)
        dY = torch.from_numpy(Y0).cuda()
        dg.dgsp_spmm_csr_axpby(300, 50, 2, 0, dE.rowptr, dE.colidx, dE.vals, torch.zeros((50, 2), device="cuda:0"), dY,
                               7.0, 0.5, algo, dE.features)
        torch.cuda.synchronize()
        assert np.array_equal(dY.cpu().numpy(), (np.float32(0.5) * Y0))


def test_plain_c_caller_of_the_library():
    """The C-ABI from a C program (built by the package's build step): all four kernels and the
    adaptive call against a host loop; the program's exit code says whether every result was in bound."""
    import subprocess
    from paper_2106_16064_amd import build
    assert build.EXAMPLE.exists(), "run `python -m paper_2106_16064_amd.build` first"
    res = subprocess.run([str(build.EXAMPLE)], capture_output=True, text=True, timeout=120)
    print(res.stdout)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.count(" ok") == 5


def test_matrix_that_is_already_on_the_device(dg):
    """CSR arrays held by a torch sparse tensor (int64 indices) are taken over without a trip to the host:
    statistics from the device pass, the adaptive call on top."""
    import torch
    A = wl.rmat_csr(scale=13, avg_degree=8, seed=77)
    t = torch.sparse_csr_tensor(torch.from_numpy(A.rowptr.astype(np.int64)), torch.from_numpy(A.colidx.astype(np.int64)),
                                torch.from_numpy(A.vals), size=(A.M, A.K)).cuda()
    dA = dg.DeviceCsr.from_torch_sparse_csr(t)
    host = dg.dgsp_features_from_csr_host(A.M, A.K, A.rowptr, A.colidx)
    assert (dA.features.nnz, dA.features.max_row, dA.features.stdv_row, dA.features.col_span) == \
           (host.nnz, host.max_row, host.stdv_row, host.col_span)
    for N in (1, 8, 32):
        X = wl.dense_matrix(A.K, N, "uniform", seed=N)
        Y = dA.spmm(torch.from_numpy(X).cuda())
        yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
        ok, worst = oracle.within_bound(Y.cpu().numpy(), yref, bnd, TOL)
        assert ok, (N, worst)


def test_gradient_when_the_matrix_lives_on_the_device_only(dg):
    """The operator built from device arrays: its transpose is made on the GPU and must hold exactly the arrays
    the host transpose gives; forward and gradient against the oracle."""
    import torch
    from paper_2106_16064_amd.autograd import SparseOperator, transpose_csr
    A = wl.rmat_csr(scale=12, avg_degree=9, seed=21)
    dA = dg.DeviceCsr.from_device(A.M, A.K, torch.from_numpy(A.rowptr).cuda(), torch.from_numpy(A.colidx).cuda(),
                                  torch.from_numpy(A.vals).cuda())
    op = SparseOperator(dA)
    T = transpose_csr(A)
    assert np.array_equal(op.bwd.rowptr.cpu().numpy(), T.rowptr) and np.array_equal(op.bwd.colidx.cpu().numpy(), T.colidx)
    assert np.array_equal(op.bwd.vals.cpu().numpy(), T.vals) and (op.bwd.M, op.bwd.K) == (A.K, A.M)
    N = 8
    X = wl.dense_matrix(A.K, N, "normal", seed=5)
    Gy = wl.dense_matrix(A.M, N, "uniform", seed=6)
    dX = torch.from_numpy(X).cuda().requires_grad_(True)
    Y = op(dX)
    Y.backward(torch.from_numpy(Gy).cuda())
    yref, bnd = oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X)
    ok, worst = oracle.within_bound(Y.detach().cpu().numpy(), yref, bnd, TOL)
    assert ok, worst
    gref, gbnd = oracle.spmm_ref(T.M, T.K, N, T.rowptr, T.colidx, T.vals, Gy)
    ok, worst = oracle.within_bound(dX.grad.cpu().numpy(), gref, gbnd, TOL)
    assert ok, worst


# ------------------------------------------------------------------ widths that are no multiple of the vector width
@pytest.mark.parametrize("N", [3, 5, 6, 7, 9, 41, 47, 63, 65, 66, 67, 129, 130, 257, 300])
def test_widths_that_are_no_multiple_of_four(dg, N):
    """The sequential kernels give a lane four columns and let the last lane of a row re-use columns of its
    neighbour: on a matrix with hub rows (partial sums meet through LDS slots and atomic adds) and many empty
    rows, plain and scaled (beta != 0 reads the old Y, which the neighbour may already have replaced), and on
    a view one float into a wider buffer (rows start at odd dword addresses)."""
    import torch
    A = wl.rmat_csr(scale=12, avg_degree=14, seed=N)
    X = wl.dense_matrix(A.K, N, "normal", seed=N)
    ref = check(dg, A, X, x_offset=1, y_offset=3)
    yref, bnd = ref
    Y0 = wl.dense_matrix(A.M, N, "uniform", seed=N + 1)
    alpha, beta = -1.5, 0.75
    want = alpha * yref + beta * Y0.astype(np.float64)
    bound = abs(alpha) * bnd + abs(beta) * np.abs(Y0.astype(np.float64))
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).cuda()
    for algo in (0, 1, 2, 3, dg.AUTO):
        print(f"[case] ragged axpby N={N} algo={algo}", flush=True)
        dY = torch.from_numpy(Y0).cuda()
        dg.dgsp_spmm_csr_axpby(A.M, A.K, N, A.nnz, dA.rowptr, dA.colidx, dA.vals, dX, dY, alpha, beta, algo, dA.features)
        torch.cuda.synchronize()
        ok, worst = oracle.within_bound(dY.cpu().numpy(), want, bound, TOL)
        assert ok, f"algo {algo}: worst |err|/bound = {worst:.3e}"
