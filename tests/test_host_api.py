"""Host-side checks that need no GPU: the library loads, exports what the header
declares, and the host functions (features, selection rules) behave."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2106_16064_amd import binding as dg
from paper_2106_16064_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dgsp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dgsp_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = dg.lib()
    names = declared_symbols()
    assert set(names) == set(dg.EXPORTS), "binding.EXPORTS and include/dgsp.h disagree"
    for name in names:
        assert getattr(L, name) is not None


def test_names_and_status_strings():
    assert [dg.dgsp_algo_name(a) for a in (0, 1, 2, 3, -1)] == ["rs_sr", "rs_pr", "nb_sr", "nb_pr", "auto"]
    assert dg.dgsp_algo_name(99) == "unknown"
    assert dg.dgsp_status_string(0) == "ok" and "invalid" in dg.dgsp_status_string(1)


@pytest.mark.parametrize("A", [wl.poisson_csr(4096, 4096, 8.0, 0), wl.rmat_csr(12, 16, seed=0),
                               wl.stencil27_csr(8), wl.sweep_csr(1 << 12, 16, "zipf", 1),
                               wl.csr_from_lens([0, 0, 0], 4)], ids=lambda a: a.name)
def test_features_match_the_oracle_statistics(A):
    f = dg.dgsp_features_from_rowptr_host(A.M, A.K, A.rowptr)
    want = oracle.row_features(A.rowptr)
    assert (f.M, f.K, f.nnz, f.max_row, f.min_row) == (A.M, A.K, A.nnz, want["max_row"], want["min_row"])
    assert f.avg_row == pytest.approx(want["avg_row"], rel=1e-14, abs=0)
    assert f.stdv_row == pytest.approx(want["stdv_row"], rel=1e-12, abs=1e-12)
    cv = want["stdv_row"] / want["avg_row"] if want["avg_row"] else 0.0
    assert f.cv_row == pytest.approx(cv, rel=1e-12, abs=1e-12)


def test_features_reject_bad_rowptr():
    L = dg.lib()
    f = dg.Features()
    bad = np.array([0, 3, 2], np.int32)
    assert L.dgsp_features_from_rowptr_host(2, 4, bad.ctypes.data, ctypes.byref(f)) == dg.ERR_INVALID_ARG
    bad0 = np.array([1, 3, 4], np.int32)
    assert L.dgsp_features_from_rowptr_host(2, 4, bad0.ctypes.data, ctypes.byref(f)) == dg.ERR_INVALID_ARG
    assert L.dgsp_features_from_rowptr_host(-1, 4, bad.ctypes.data, ctypes.byref(f)) == dg.ERR_INVALID_ARG
    assert L.dgsp_features_from_rowptr_host(2, 4, bad.ctypes.data, None) == dg.ERR_INVALID_ARG
    z = np.zeros(1, np.int32)
    assert L.dgsp_features_from_rowptr_host(0, 4, z.ctypes.data, ctypes.byref(f)) == dg.OK and f.nnz == 0


def feat(avg, cv, M=1000):
    f = dg.Features()
    f.M, f.K, f.nnz = M, M, int(avg * M)
    f.avg_row, f.stdv_row, f.cv_row = avg, avg * cv, cv
    f.max_row = int(avg * (1 + 3 * cv)) + 1
    return f


def test_selection_rules_follow_the_decision_tree():
    """Section 2.2: N decides parallel vs sequential; avg_row (parallel side) and
    stdv_row/avg_row (sequential side) decide whether to balance."""
    saved = dg.dgsp_get_thresholds()
    try:
        t = dg.Thresholds(4, 32.0, 1e30, 1.0, 0.0, 2**62, 0.0, 0, 0, 0, 0.0, 0.0, 0, 0, 0.0)   # the paper's rule verbatim (no added guards)
        dg.dgsp_set_thresholds(t)
        got = dg.dgsp_get_thresholds()
        assert (got.n_parallel_max, got.pr_avg_row_min, got.sr_cv_min) == (4, 32.0, 1.0)
        for N in (1, 2, 4):
            assert dg.dgsp_select_algo(feat(64, 0.1), N) == dg.RS_PR      # long rows: row-split
            assert dg.dgsp_select_algo(feat(64, 5.0), N) == dg.RS_PR      # paper ignores skew here
            assert dg.dgsp_select_algo(feat(4, 0.1), N) == dg.NB_PR       # short rows: balanced
        for N in (5, 8, 128, 512):
            assert dg.dgsp_select_algo(feat(64, 0.1), N) == dg.RS_SR
            assert dg.dgsp_select_algo(feat(4, 0.9), N) == dg.RS_SR
            assert dg.dgsp_select_algo(feat(4, 1.1), N) == dg.NB_SR       # uneven rows: balanced
        t.pr_cv_max = 0.5                                                  # the added skew guard
        dg.dgsp_set_thresholds(t)
        assert dg.dgsp_select_algo(feat(64, 5.0), 1) == dg.NB_PR
        assert dg.dgsp_select_algo(feat(64, 0.1), 1) == dg.RS_PR
        t.sr_stdv_min = 30.0                                               # the added short-row guard
        dg.dgsp_set_thresholds(t)
        assert dg.dgsp_select_algo(feat(4, 1.5), 64) == dg.RS_SR           # stdv 6: rows too short to matter
        assert dg.dgsp_select_algo(feat(64, 1.5), 64) == dg.NB_SR          # stdv 96
        t.n_parallel_max = 8
        dg.dgsp_set_thresholds(t)
        assert dg.dgsp_select_algo(feat(64, 0.1), 8) == dg.RS_PR
        t.pr_nnz_max = 50_000                                              # the added size guard
        dg.dgsp_set_thresholds(t)
        assert dg.dgsp_select_algo(feat(64, 0.1, M=1000), 1) == dg.NB_PR   # 64 000 entries: second launch pays
        assert dg.dgsp_select_algo(feat(64, 0.1, M=500), 1) == dg.RS_PR    # 32 000 entries
        assert dg.dgsp_select_algo(feat(64, 0.1, M=1000), 64) == dg.RS_SR  # sequential side unaffected
        t.short_avg_row_max, t.short_max_row_max = 20.0, 64                # the added short-row rule
        dg.dgsp_set_thresholds(t)
        f = feat(4, 0.5); f.max_row = 16
        assert dg.dgsp_select_algo(f, 2) == dg.RS_SR                       # every row short: one lane per row
        assert dg.dgsp_select_algo(f, 64) == dg.RS_SR                      # ... at every width
        f.max_row = 400
        assert dg.dgsp_select_algo(f, 2) != dg.RS_SR                       # one long row: back to the tree
        f = feat(40, 0.1); f.max_row = 50
        assert dg.dgsp_select_algo(f, 2) != dg.RS_SR                       # rows not short on average
        t.wide_parallel_n, t.n_parallel_max = 8, 4                         # the added eight-column rule
        dg.dgsp_set_thresholds(t)
        assert dg.dgsp_select_algo(feat(64, 1.5), 8) == dg.NB_PR           # balanced, and 8 columns fit one lane
        assert dg.dgsp_select_algo(feat(64, 1.5), 16) == dg.NB_SR
        assert dg.dgsp_select_algo(feat(64, 1.5), 7) == dg.NB_PR           # 5, 6, 7 too: its two groups of four overlap
        assert dg.dgsp_select_algo(feat(64, 0.1), 8) == dg.RS_SR           # even rows: row-split as before
        t.big_x_bytes_min, t.big_x_cv_max, t.big_x_avg_row_max = 6_000_000, 0.2, 64.0     # the added large-X rule
        t.pr_nnz_max = 2**62
        dg.dgsp_set_thresholds(t)
        f = feat(30, 0.1, M=1 << 20); f.col_span = 0.9                     # K * 4 * 4 = 16 MB, rows alike, columns spread
        assert dg.dgsp_select_algo(f, 4) == dg.RS_SR and dg.dgsp_select_algo(f, 2) == dg.RS_SR
        assert dg.dgsp_select_algo(f, 1) == dg.NB_PR                       # 4 MB: X still fits an L2
        f.col_span = 0.01
        assert dg.dgsp_select_algo(f, 4) == dg.NB_PR                       # banded: neighbours share X anyway
        f.col_span = 0.0
        assert dg.dgsp_select_algo(f, 4) == dg.NB_PR                       # span unknown: the rule stays out
        f = feat(30, 0.6, M=1 << 20); f.col_span = 0.9
        assert dg.dgsp_select_algo(f, 4) == dg.NB_PR                       # uneven rows
        f = feat(100, 0.1, M=1 << 20); f.col_span = 0.9
        assert dg.dgsp_select_algo(f, 4) == dg.RS_PR                       # long rows: the tree's parallel side
        t.short_min_waves = 2048                                           # short rows need enough of them
        dg.dgsp_set_thresholds(t)
        f = feat(4, 0.5, M=1 << 18); f.max_row = 16
        assert dg.dgsp_select_algo(f, 2) == dg.RS_SR                       # 4096 waves of one row per lane
        f = feat(4, 0.5, M=1 << 16); f.max_row = 16
        assert dg.dgsp_select_algo(f, 2) == dg.NB_PR                       # 1024 waves: back to the tree
        assert dg.dgsp_select_algo(f, 32) == dg.RS_SR                      # eight lanes per row: 8192 waves
        t.pr_small_nnz_max, t.pr_small_cv_max = 2_000_000, 0.6             # the added small-matrix rule
        dg.dgsp_set_thresholds(t)
        assert dg.dgsp_select_algo(f, 2) == dg.RS_PR                       # 262 144 entries, rows about alike
        f = feat(26, 0.13, M=64000); f.max_row = 27
        assert dg.dgsp_select_algo(f, 1) == dg.RS_PR and dg.dgsp_select_algo(f, 4) == dg.RS_PR
        assert dg.dgsp_select_algo(f, 8) == dg.RS_SR                       # sequential side unaffected
        f = feat(26, 2.0, M=64000)
        assert dg.dgsp_select_algo(f, 1) == dg.NB_PR                       # uneven rows stay balanced
        f = feat(26, 0.13, M=1 << 20); f.col_span = 0.01
        assert dg.dgsp_select_algo(f, 1) == dg.NB_PR                       # 27 million entries: the second launch pays
        L = dg.lib()
        assert L.dgsp_select_algo(None, 4) == dg.AUTO
        assert dg.dgsp_select_algo(feat(4, 1), 0) == dg.AUTO
    finally:
        dg.dgsp_set_thresholds(saved)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(dg, "_lib", None)
    monkeypatch.setattr(dg, "LIB_PATH", tmp_path / "libdgsp.so")
    with pytest.raises(dg.DgspError):
        dg.lib()


def test_column_span_feature():
    S = wl.stencil27_csr(10)
    f = dg.dgsp_features_from_csr_host(S.M, S.K, S.rowptr, S.colidx)
    # interior rows span 2*(n*n + n + 1) + 1 columns of n^3
    assert 0.1 < f.col_span < 2 * (100 + 10 + 1 + 1) / 1000
    assert (f.nnz, f.max_row) == (S.nnz, 27)
    R = wl.poisson_csr(2000, 2000, 16.0, seed=1)
    fr = dg.dgsp_features_from_csr_host(R.M, R.K, R.rowptr, R.colidx)
    assert fr.col_span > 0.7
    # unsorted rows give the same span
    rng = np.random.default_rng(0)
    c2 = R.colidx.copy()
    for i in range(R.M):
        s, e = R.rowptr[i], R.rowptr[i + 1]
        c2[s:e] = rng.permutation(c2[s:e])
    fu = dg.dgsp_features_from_csr_host(R.M, R.K, R.rowptr, c2)
    assert fu.col_span == pytest.approx(fr.col_span, rel=1e-12)
    # by hand: rows {1,3}, {}, {5} of K = 10 -> ((3-1+1) + 1) / 2 / 10
    f3 = dg.dgsp_features_from_csr_host(3, 10, np.array([0, 2, 2, 3], np.int32), np.array([1, 3, 5], np.int32))
    assert f3.col_span == pytest.approx(0.2)
    assert dg.dgsp_features_from_rowptr_host(3, 10, np.array([0, 2, 2, 3], np.int32)).col_span == 0.0


def test_c_example_builds_and_links_against_the_library():
    """The plain-C caller compiles with gcc against include/dgsp.h and links to libdgsp.so (running it needs a GPU)."""
    from paper_2106_16064_amd import build
    exe = build.build_c_example(verbose=False)
    assert exe.exists() and exe.stat().st_size > 0


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys, os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "single-GPU" in (r.stderr + r.stdout)


def test_default_thresholds_and_their_effect_on_benchmark_shapes():
    """The shipped rules on the statistics of the benchmark's matrices (computed here from the generators):
    R-MAT -> balanced kernels, stencil -> balanced parallel up to N = 4 and row-split sequential at 8,
    equal rows of random columns -> row-split sequential once X outgrows an L2."""
    t = dg.dgsp_get_thresholds()
    assert (t.n_parallel_max, t.wide_parallel_n, t.big_x_bytes_min) == (4, 8, 6_000_000)
    R = wl.rmat_csr(14, 16, seed=0)
    f = dg.dgsp_features_from_csr_host(R.M, R.K, R.rowptr, R.colidx)
    assert [dg.dgsp_select_algo(f, n) for n in (1, 4, 8, 32)] == [dg.NB_PR, dg.NB_PR, dg.NB_PR, dg.NB_SR]
    S = wl.stencil27_csr(24)
    f = dg.dgsp_features_from_csr_host(S.M, S.K, S.rowptr, S.colidx)
    f.nnz = 55_742_968                       # as large as the benchmark's grid: beyond the single-launch size guard
    assert [dg.dgsp_select_algo(f, n) for n in (1, 2, 4, 8)] == [dg.NB_PR, dg.NB_PR, dg.NB_PR, dg.RS_SR]
    E = wl.sweep_csr(1 << 12, 27, "fixed", 0)
    f = dg.dgsp_features_from_csr_host(E.M, E.K, E.rowptr, E.colidx)
    assert f.cv_row == 0.0 and f.col_span > 0.8
    assert dg.dgsp_select_algo(f, 4) == dg.RS_PR        # 110 592 entries of equal rows: a small matrix, one launch
    f.nnz = 27 << 20                                    # as many rows as the size study's: the tree decides
    assert dg.dgsp_select_algo(f, 4) == dg.NB_PR        # 4096 columns: X is 64 KB
    f.K = 1 << 20                                       # the same rows over 2^20 columns: X is 16 MB at N = 4
    assert dg.dgsp_select_algo(f, 4) == dg.RS_SR and dg.dgsp_select_algo(f, 1) == dg.NB_PR
    small = wl.stencil27_csr(24)                        # 13 824 rows: short of rows for one lane per row
    f = dg.dgsp_features_from_csr_host(small.M, small.K, small.rowptr, small.colidx)
    assert [dg.dgsp_select_algo(f, n) for n in (1, 4, 8)] == [dg.RS_PR, dg.RS_PR, dg.RS_SR]


def test_the_benchmark_mirror_of_the_rules_agrees_with_the_library():
    """bench.py scores recorded timings with a Python copy of the selection rules (`rules_choose`, used by
    `--suite fit`); the losses it reports are only worth something if that copy picks what `dgsp_select_algo`
    picks.  Seeded random row statistics around every threshold, every N of the sweeps."""
    import sys
    from pathlib import Path
    sys.path.insert(0, str(Path(__file__).resolve().parents[1]))
    import bench
    t = dg.dgsp_get_thresholds()
    td = {name: getattr(t, name) for name in bench.THRESHOLD_NAMES}
    rng = np.random.default_rng(7)
    names = {dg.RS_SR: "rs_sr", dg.RS_PR: "rs_pr", dg.NB_SR: "nb_sr", dg.NB_PR: "nb_pr"}
    checked = 0
    for _ in range(4000):
        M = int(2 ** rng.uniform(8, 22))
        K = int(2 ** rng.uniform(8, 22))
        avg = float(rng.choice([0.2, 3.9, 4.0, 16.0, 19.9, 20.1, 27.0, 47.9, 48.1, 64.0, 100.0]) * rng.uniform(0.9, 1.1))
        cv = float(rng.choice([0.0, 0.04, 0.06, 0.19, 0.21, 0.29, 0.31, 0.59, 0.61, 1.3, 9.0]))
        nnz = max(1, int(M * avg))
        f = dg.Features()
        f.M, f.K, f.nnz = M, K, nnz
        f.avg_row, f.cv_row, f.stdv_row = nnz / M, cv, cv * (nnz / M)
        f.max_row = int(rng.choice([4, 27, 63, 64, 65, 200, 40000]))
        f.min_row = 0
        f.col_span = float(rng.choice([0.0, 0.01, 0.49, 0.51, 1.0]))
        for N in (1, 2, 3, 4, 5, 8, 9, 16, 31, 32, 64, 100, 128, 256, 512):
            rec = {"N": N, "M": M, "K": K, "nnz": nnz, "avg_row": f.avg_row, "cv_row": f.cv_row, "max_row": f.max_row,
                   "col_span": f.col_span}
            assert bench.rules_choose(rec, td) == names[dg.dgsp_select_algo(f, N)], (rec, td)
            checked += 1
    assert checked == 60000
