#!/usr/bin/env python3
"""Benchmark of the CSR SpMV/SpMM hot path on one MI355X.

Default run (what the driver calls):
    python bench.py --gpus 1 --steps K --warmup W
times K "steps" of the power-law SpMV configuration (R-MAT 2^20 vertices,
average degree 16, N = 1).  One step = the whole hot path once: the selection
rules on the matrix's precomputed row statistics, then the chosen kernel
(through ``dgsp_spmm_csr_auto``).  Inputs are resident in device memory before
the timed region; successive steps rotate over several copies of (A, X, Y) so
that every step streams its operands from HBM rather than from the 256 MB
Infinity Cache (one copy of this workload, ~141 MB, would fit).  Prints ONE
JSON line.

Other suites (for the tables under profiles/; each still prints one JSON line
and writes its per-cell records under RESULTS_DIR):
    --suite configs   every kernel on the R-MAT and stencil configurations
    --suite sweep     the 24-matrix x 10-N selector sweep (loss vs best kernel)
    --suite kernel --workload W --n N --algo A   one kernel in a loop (for rocprofv3)
    --suite size      all four kernels on banded and random matrices of growing size, N <= 8
    --suite ablation  each optimisation against the kernel without it, on 27 R-MAT matrices
    --suite tiny      the launch-bound 4096^2 configuration, eager launches against HIP graph replay
    --suite fit       fits the selector thresholds on a finished sweep (no GPU)
    --suite widths    the adaptive call at 34 dense widths from 1 to 128 on three matrices
    --suite holdout   the shipped selection rules scored on matrices they were not fitted on
    --suite layouts   the balanced sequential kernel's wide-N column layouts on the GNN configuration
    --suite gather    dgsp_gather_probe on synthetic index patterns (what a gather costs per lane layout)
    --suite colranges the GNN configuration as passes over column ranges of A (Y accumulated pass by pass)
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
CACHE_BYTES = 256e6 + 32e6     # Infinity Cache + 8 x 4 MB L2: what rotation has to exceed
RESULTS_DIR = "gpurun_out"     # per-cell records of the suites

# HBM bytes per launch of the dominant kernel, measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE in
# separate runs, scaled by the same counters on dgsp_copy_f32).  These are NOT measured by this run: they are
# copied from the named summaries under profiles/, taken on the same build, and the JSON line says so
# ("traffic_source").  A cell without an entry reports null.
_TRAFFIC_SOURCE = "profiles/selected_kernels_time_traffic_occupancy.md (rocprofv3 FETCH_SIZE + WRITE_SIZE per launch, scaled by the copy kernel)"
MEASURED_TRAFFIC = {
    # "kernel/workload/N": (bytes fetched + bytes written per launch of the main kernel, source)
    "nb_pr/rmat_spmv/N1": (169.3e6 + 5.1e6, _TRAFFIC_SOURCE),
    "nb_sr/rmat_gnn/N128": (5376.8e6 + 644.3e6, _TRAFFIC_SOURCE),
    "nb_sr/rmat_gnn/N32": (1147.9e6 + 161.1e6, _TRAFFIC_SOURCE),
    "nb_pr/stencil/N1": (505.6e6 + 8.7e6, _TRAFFIC_SOURCE),
    "rs_sr/stencil/N8": (619.6e6 + 67.1e6, _TRAFFIC_SOURCE),
    "rs_pr/uniform64/N4": (272.7e6 + 5.2e6, _TRAFFIC_SOURCE),
}


def algorithmic_bytes(A, N):
    """Bytes the method has to move once: 8 per stored entry (column index and
    value), rowptr, every touched row of X once, Y once."""
    return 8 * A.nnz + 4 * (A.M + 1) + 4 * A.k_touched() * N + 4 * A.M * N


_MATRIX_CACHE = {}


def make_workload(name, n):
    """(A, X, label) of a named benchmark configuration; A is cached per name."""
    from paper_2106_16064_amd import workloads as wl
    gens = {
        "rmat_spmv": (lambda: wl.rmat_csr(20, 16, seed=0, values="uniform01"), "uniform",
                      "power-law SpMV/SpMM: R-MAT 2^20 vertices, avg degree 16, U(0,1) values"),
        "rmat_gnn": (lambda: wl.rmat_csr(20, 16, seed=0, values="rownorm"), "normal",
                     "GNN-style SpMM: R-MAT 2^20 vertices, avg degree 16, row-normalised"),
        "stencil": (lambda: wl.stencil27_csr(128, seed=0), "uniform", "27-point stencil on 128^3"),
        "tiny": (lambda: wl.poisson_csr(4096, 4096, 8.0, seed=0), "uniform", "tiny SpMM: 4096^2 Poisson(8)"),
        "uniform64": (lambda: wl.sweep_csr(1 << 18, 64, "fixed", 0), "uniform",
                      "sweep matrix: 2^18 rows of exactly 64 uniform-random columns"),
    }
    if name not in gens:
        raise SystemExit(f"unknown workload {name}")
    gen, xdist, label = gens[name]
    if name not in _MATRIX_CACHE:
        other = {"rmat_gnn": "rmat_spmv", "rmat_spmv": "rmat_gnn"}.get(name)
        if other in _MATRIX_CACHE:
            # the two R-MAT configurations share one pattern (same seed, same draws): only the values differ,
            # and the generator draws them after the pattern, so regenerating would give the same arrays
            P = _MATRIX_CACHE[other]
            lens = P.row_lengths()
            vals = ((1.0 / np.repeat(lens, lens).astype(np.float64)).astype(np.float32) if name == "rmat_gnn"
                    else gen().vals)
            new = wl.CsrMatrix(P.M, P.K, P.rowptr, P.colidx, vals, name, dict(P.meta, values=name))
            _MATRIX_CACHE.clear()
            _MATRIX_CACHE[name] = new
        else:
            _MATRIX_CACHE.clear()          # one big matrix at a time on the host
            _MATRIX_CACHE[name] = gen()
    A = _MATRIX_CACHE[name]
    return A, wl.dense_matrix(A.K, n, xdist, seed=0), f"{label}, N={n}"


class Rotation:
    """R device copies of (A, X, Y): step i uses copy i % R."""

    def __init__(self, A, X, copies=None, device="cuda:0"):
        import torch
        from paper_2106_16064_amd import binding as dg
        self.A, self.N = A, X.shape[1]
        foot = algorithmic_bytes(A, self.N)
        if copies is None:
            copies = int(min(8, max(2, -(-3 * CACHE_BYTES // foot))))
        self.copies = copies
        base = dg.DeviceCsr(A, device)
        self.mats = [base]
        for _ in range(copies - 1):
            m = dg.DeviceCsr.__new__(dg.DeviceCsr)
            m.M, m.K, m.nnz, m.features = base.M, base.K, base.nnz, base.features
            m.rowptr, m.colidx, m.vals = base.rowptr.clone(), base.colidx.clone(), base.vals.clone()
            self.mats.append(m)
        x0 = torch.from_numpy(X).to(device)
        self.X = [x0] + [x0.clone() for _ in range(copies - 1)]
        self.Y = [torch.empty((A.M, self.N), dtype=torch.float32, device=device) for _ in range(copies)]

    def step(self, i, algo, warm=False):
        j = 0 if warm else i % self.copies
        self.mats[j].spmm(self.X[j], algo=algo, Y=self.Y[j])

    def ablation(self, i, algo, switches):
        """The call with optimisations switched off (measurement aid)."""
        from paper_2106_16064_amd import binding as dg
        j = i % self.copies
        m = self.mats[j]
        dg.dgsp_spmm_csr_ablation(m.M, m.K, self.N, m.nnz, m.rowptr, m.colidx, m.vals, self.X[j], self.Y[j],
                                  algo, switches, m.features)

    def phase(self, i, algo, phase):
        """One launch of a call (measurement aid): the prepare step or the main kernel alone."""
        from paper_2106_16064_amd import binding as dg
        j = i % self.copies
        m = self.mats[j]
        dg.dgsp_spmm_csr_phase(m.M, m.K, self.N, m.nnz, m.rowptr, m.colidx, m.vals, self.X[j], self.Y[j],
                               algo, phase, m.features)


def time_steps(rot, algo, steps, warmup, warm=False):
    """Wall-clock ms per step over `steps` back-to-back launches."""
    import torch
    spin_up(None, lambda i: rot.step(i, algo, warm))
    for i in range(warmup):
        rot.step(i, algo, warm)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        rot.step(i, algo, warm)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


SPIN_UP_MS = 40.0


def spin_up(fn_before, fn_timed, ms=SPIN_UP_MS):
    """Untimed launches for `ms` of wall time before a measurement: while the host builds the next matrix the device
    idles and its clocks fall, and the first few milliseconds of work afterwards run up to 5 % slower (27-point
    stencil, N = 1: 138 us in the first measurement after a second of idling, 131 us in the next four and after
    a spin-up)."""
    import torch
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < ms * 1e-3:
        if fn_before:
            fn_before(i)
        fn_timed(i)
        i += 1
        if i % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()


def time_events(fn_before, fn_timed, steps, warmup):
    """Per-launch durations (ms) of fn_timed(i), bracketed by HIP events on the
    launch stream; fn_before(i) runs untimed just before each launch."""
    import torch
    spin_up(fn_before, fn_timed)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i in range(warmup):
        if fn_before:
            fn_before(i)
        fn_timed(i)
    torch.cuda.synchronize()
    for i in range(steps):
        if fn_before:
            fn_before(i)
        evs[i][0].record()
        fn_timed(i)
        evs[i][1].record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in evs]


def time_event_batches(fn_before, fn_timed, batch, batches, warmup):
    """Mean duration (ms) of one fn_timed launch: each HIP-event pair brackets `batch` back-to-back
    launches (i = 0..batch-1), so the pair's own cost is spread over the batch; fn_before(i) runs
    untimed for every i before the batch starts."""
    import torch
    spin_up(fn_before, fn_timed)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(batches)]
    for b in range(warmup + batches):
        if fn_before:
            for i in range(batch):
                fn_before(i)
        if b >= warmup:
            evs[b - warmup][0].record()
        for i in range(batch):
            fn_timed(i)
        if b >= warmup:
            evs[b - warmup][1].record()
    torch.cuda.synchronize()
    return [a.elapsed_time(c) / batch for a, c in evs]


def median(v):
    s = sorted(v)
    return s[len(s) // 2]


def copy_bandwidth(nbytes=1 << 30, reps=10):
    """Achieved GB/s (read + write) of the plain streaming copy kernel."""
    import torch
    from paper_2106_16064_amd import binding as dg
    n = nbytes // 4
    src = torch.empty(n, dtype=torch.float32, device="cuda:0").normal_()
    dst = torch.empty_like(src)
    ms = time_events(None, lambda i: dg.dgsp_copy_f32(dst, src, n), reps, 3)
    return 2 * nbytes / (median(ms) * 1e-3) / 1e9


def floor_probes(rot):
    """Times (ms) of the committed floor probes on this workload's own arrays: the memory side of the kernels
    with no row logic (dgsp_floor_probe).  N <= 4: stream + gather + multiply-add (and the bare gather at N = 1);
    N a multiple of 4 from 8 on: the whole-row gather of the sequential kernels."""
    import torch
    from paper_2106_16064_amd import binding as dg
    N, K = rot.N, rot.A.K
    out = {}
    modes = []
    if N == 1:
        modes.append(("gather_only_ms", dg.PROBE_GATHER))
    if N in (1, 2, 4):
        modes.append(("stream_gather_fma_ms", dg.PROBE_STREAM_GATHER_FMA))
    if N >= 8 and N % 4 == 0:
        modes.append(("row_gather_ms", dg.PROBE_ROW_GATHER))
    for key, mode in modes:
        buf = torch.empty(dg.dgsp_floor_probe_out_len(mode, N), dtype=torch.float32, device="cuda:0")
        ms = time_events(None, lambda i: dg.dgsp_floor_probe(mode, K, N, rot.mats[i % rot.copies].colidx,
                                                             rot.mats[i % rot.copies].vals, rot.X[i % rot.copies], buf),
                         2 * rot.copies + 6, 3)
        out[key] = median(ms)
    return out


def sampled_parity(A, X, Y, rows=20000, seed=0, tol=1e-5):
    """The oracle on a seeded sample of rows (plus the longest row and both ends), against the same rows of the
    GPU result Y (a host array)."""
    import oracle
    rng = np.random.default_rng(seed)
    lens = A.row_lengths()
    pick = np.unique(np.concatenate([rng.integers(0, A.M, size=min(rows, A.M)), [int(lens.argmax()), 0, A.M - 1]]))
    plen = lens[pick].astype(np.int64)
    rp = np.zeros(pick.size + 1, dtype=np.int64)
    np.cumsum(plen, out=rp[1:])
    idx = np.repeat(A.rowptr[pick].astype(np.int64) - rp[:-1], plen) + np.arange(int(rp[-1]))
    N = X.shape[1]
    yref, bnd = oracle.spmm_ref(pick.size, A.K, N, rp.astype(np.int32), A.colidx[idx], A.vals[idx], X)
    ok, worst = oracle.within_bound(Y[pick], yref, bnd, tol)
    return {"ok": bool(ok), "worst_err_over_bound": worst, "tol": tol, "rows_checked": int(pick.size)}


def measure_cell(name, n, steps, warmup, full_parity=False):
    """One configuration through the adaptive call: whole-call time over rotated buffers, the selected kernel's
    main launch alone (HIP events on the launch stream), its floors, its roofline, parity against the oracle."""
    import torch
    from paper_2106_16064_amd import binding as dg
    A, X, label = make_workload(name, n)
    rot = Rotation(A, X)
    chosen = dg.dgsp_select_algo(rot.mats[0].features, n)
    sel = dg.dgsp_algo_name(chosen)
    ms_cold = time_steps(rot, dg.AUTO, steps, warmup, warm=False)
    batches = max(2, steps // rot.copies)
    ev = time_event_batches(lambda i: rot.phase(i, chosen, dg.PHASE_PREPARE),
                            lambda i: rot.phase(i, chosen, dg.PHASE_MAIN), rot.copies, batches,
                            max(1, warmup // rot.copies))
    ev_ms = sum(ev) / len(ev)
    floors = floor_probes(rot)
    rot.step(0, dg.AUTO)
    torch.cuda.synchronize()
    Y = rot.Y[0].cpu().numpy()
    if full_parity:
        import oracle
        yref, bnd = oracle.spmm_ref(A.M, A.K, n, A.rowptr, A.colidx, A.vals, X)
        ok, worst = oracle.within_bound(Y, yref, bnd, 1e-5)
        parity = {"ok": bool(ok), "worst_err_over_bound": worst, "tol": 1e-5, "rows_checked": A.M}
    else:
        parity = sampled_parity(A, X, Y)
    bytes_alg = algorithmic_bytes(A, n)
    achieved = bytes_alg / (ev_ms * 1e-3) / 1e9
    traffic, source = MEASURED_TRAFFIC.get(f"{sel}/{name}/N{n}", (None, None))
    cell = {
        "workload": label, "M": A.M, "K": A.K, "nnz": A.nnz, "N": n, "buffer_rotation": rot.copies,
        "selected_kernel": sel, "ms_per_step": ms_cold,
        "GFLOPs": 2.0 * A.nnz * n / (ms_cold * 1e-3) / 1e9,
        "algorithmic_bytes": bytes_alg, "effective_GBps": bytes_alg / (ms_cold * 1e-3) / 1e9,
        "pct_hbm_peak": 100.0 * bytes_alg / (ms_cold * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": source,
                     "kernel": f"dgsp::{sel}_kernel (main launch alone; HIP events on the launch stream around "
                               f"{len(ev)} batches of {rot.copies} back-to-back launches, one per buffer set)",
                     "algorithmic_bytes": bytes_alg, "launch_ms": ev_ms, "floors_ms": floors},
        "parity": parity,
    }
    return cell, rot, A, X


def cpu_baseline(A, X, budget_s=8.0):
    """The CPU oracle (test infrastructure, never tuned) on the same workload."""
    import oracle
    N = X.shape[1]
    oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X, with_bound=False)   # warm-up, builds the .so
    times = []
    t_start = time.perf_counter()
    while len(times) < 3 or (time.perf_counter() - t_start < budget_s and len(times) < 200):
        t0 = time.perf_counter()
        oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X, with_bound=False)
        times.append(time.perf_counter() - t0)
    best = min(times)
    cores = oracle.max_threads()
    single = []
    for _ in range(2):
        t0 = time.perf_counter()
        oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X, with_bound=False, nthreads=1)
        single.append(time.perf_counter() - t0)
    oracle.spmm_ref(A.M, A.K, N, A.rowptr, A.colidx, A.vals, X, with_bound=False, nthreads=cores)   # back to all threads
    return {"value": 2.0 * A.nnz * N / best / 1e9, "unit": "GFLOP/s", "cores": cores,
            "kind": "oracle", "ms_per_pass": best * 1e3,
            "one_thread": {"value": 2.0 * A.nnz * N / min(single) / 1e9, "ms_per_pass": min(single) * 1e3},
            "effective_GBps": algorithmic_bytes(A, N) / best / 1e9,
            "sample": f"the full workload ({A.nnz} stored entries, N={N}), best of {len(times)} passes of the "
                      f"fp64 oracle incl. its input validation, OpenMP over rows"}


def variant_table(rot, steps, warmup):
    """Event-timed median ms of each of the four kernels on the rotation's workload."""
    from paper_2106_16064_amd import binding as dg
    out = {}
    for algo in dg.ALGOS:
        k = max(5, min(steps, 20))
        ms = time_events(None, lambda i: rot.step(i, algo), k, 3)
        out[dg.dgsp_algo_name(algo)] = median(ms)
    return out


# ---------------------------------------------------------------------------- suites
# The further cells of the default line: the largest single-GPU configurations of the benchmark list, which the
# bandwidth target is stated on (GNN-style SpMM at N = 128, the stencil at N = 1 and at N = 8).
FURTHER_CELLS = (("rmat_gnn", 128), ("stencil", 1), ("stencil", 8))


def run_headline(args):
    import torch
    from paper_2106_16064_amd import binding as dg
    name = args.workload or "rmat_spmv"
    N = args.n or 1
    head, rot, A, X = measure_cell(name, N, args.steps, args.warmup, full_parity=True)
    ms_cold = head["ms_per_step"]
    ms_warm = time_steps(rot, dg.AUTO, args.steps, args.warmup, warm=True)
    bytes_alg = head["algorithmic_bytes"]
    flops = 2.0 * A.nnz * N
    table = variant_table(rot, args.steps, args.warmup)
    best = min(table, key=table.get)
    sel_name = head["selected_kernel"]
    baseline = cpu_baseline(A, X)
    del rot
    torch.cuda.empty_cache()

    cells = []
    if not args.workload and not args.no_cells:
        for cname, cn in FURTHER_CELLS:
            cell, crot, _, _ = measure_cell(cname, cn, max(10, min(args.steps, 40)), min(args.warmup, 5))
            del crot
            torch.cuda.empty_cache()
            cells.append(cell)
            print(f"[cell] {cell['workload']}: {cell['selected_kernel']} {cell['ms_per_step'] * 1e3:.1f} us per call, "
                  f"main launch {cell['roofline']['launch_ms'] * 1e3:.1f} us, frac {cell['roofline']['frac']:.3f}, "
                  f"parity {'ok' if cell['parity']['ok'] else 'FAIL'}", file=sys.stderr, flush=True)

    roof = head["roofline"]
    copy_gbps = copy_bandwidth()
    for c in [head] + cells:
        # the same algorithmic bytes against what a plain copy reaches on this machine (the achievable ceiling)
        c["pct_of_measured_copy"] = 100.0 * c["effective_GBps"] / copy_gbps
        c["no_reuse_bytes"] = 8 * c["nnz"] + 4 * c["nnz"] * c["N"] + 4 * c["M"] * c["N"]
    out = {
        "metric": "SpMM GFLOP/s (2*nnz*N/t); effective HBM GB/s and selector loss alongside",
        "value": flops / (ms_cold * 1e-3) / 1e9, "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_cold,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "M": A.M, "K": A.K, "nnz": A.nnz, "N": N,
                   "buffer_rotation": head["buffer_rotation"], "selected_kernel": sel_name,
                   "why_this_workload": "the benchmark list's second configuration (power-law SpMV), the one the "
                                        "default line is defined on; the larger configurations follow under 'cells'"},
        "effective_GBps": head["effective_GBps"], "pct_hbm_peak": head["pct_hbm_peak"],
        "pct_of_measured_copy": head["pct_of_measured_copy"], "no_reuse_bytes": head["no_reuse_bytes"],
        "warm_cache": {"ms_per_step": ms_warm, "GFLOPs": flops / (ms_warm * 1e-3) / 1e9,
                       "effective_GBps": bytes_alg / (ms_warm * 1e-3) / 1e9},
        "copy_kernel_GBps": copy_gbps,
        "selector": {"chosen": sel_name, "best": best, "loss_vs_best": table[sel_name] / table[best] - 1.0,
                     "median_ms": table},
        "parity": head["parity"],
        "roofline": roof,
        "cpu_baseline": baseline,
        "cells": cells,
    }
    print(json.dumps(out))
    return 0 if head["parity"]["ok"] and all(c["parity"]["ok"] for c in cells) else 1


def run_configs(args):
    from paper_2106_16064_amd import binding as dg
    os.makedirs(RESULTS_DIR, exist_ok=True)
    cells = [("rmat_spmv", 1), ("rmat_spmv", 2), ("rmat_spmv", 4), ("rmat_gnn", 32), ("rmat_gnn", 64),
             ("rmat_gnn", 128), ("stencil", 1), ("stencil", 2), ("stencil", 4), ("stencil", 8)]
    if args.workload:
        cells = [c for c in cells if c[0] == args.workload]
    rows = []
    path = os.path.join(RESULTS_DIR, args.out or "bench_configs.jsonl")
    with open(path, "w") as fh:
        for name, n in cells:
            A, X, label = make_workload(name, n)
            rot = Rotation(A, X)
            table = variant_table(rot, args.steps, args.warmup)
            sel = dg.dgsp_algo_name(dg.dgsp_select_algo(rot.mats[0].features, n))
            best = min(table, key=table.get)
            ba = algorithmic_bytes(A, n)
            row = {"workload": label, "N": n, "nnz": A.nnz, "algorithmic_bytes": ba, "selected": sel, "best": best,
                   "loss_vs_best": table[sel] / table[best] - 1.0,
                   "kernels": {k: {"ms": v, "GFLOPs": 2.0 * A.nnz * n / v / 1e6, "GBps": ba / v / 1e6,
                                   "pct_hbm_peak": 100 * ba / v / 1e6 / HBM_PEAK_GBS} for k, v in table.items()}}
            rows.append(row)
            fh.write(json.dumps(row) + "\n")
            fh.flush()
            print(f"[configs] {name} N={n}: " + ", ".join(f"{k} {v:.3f} ms" for k, v in table.items())
                  + f" | selected {sel}, best {best}", file=sys.stderr, flush=True)
            del rot
    print(json.dumps({"suite": "configs", "cells": len(rows), "file": path}))
    return 0


def run_sweep(args):
    from paper_2106_16064_amd import binding as dg
    from paper_2106_16064_amd import workloads as wl
    os.makedirs(RESULTS_DIR, exist_ok=True)
    path = os.path.join(RESULTS_DIR, args.out or "bench_sweep.jsonl")
    M = args.sweep_m
    losses = []
    with open(path, "w") as fh:
        for A in wl.sweep_matrices(M):
            for n in wl.SWEEP_NS:
                X = wl.dense_matrix(A.K, n, "uniform", seed=0)
                rot = Rotation(A, X, copies=2)
                table = variant_table(rot, args.steps, args.warmup)
                f = rot.mats[0].features
                sel = dg.dgsp_algo_name(dg.dgsp_select_algo(f, n))
                best = min(table, key=table.get)
                loss = table[sel] / table[best] - 1.0
                losses.append(loss)
                fh.write(json.dumps({"matrix": A.name, "N": n, "M": A.M, "avg_row": f.avg_row, "cv_row": f.cv_row,
                                     "max_row": f.max_row, "nnz": A.nnz, "K": A.K, "col_span": f.col_span, "ms": table, "selected": sel,
                                     "best": best, "loss": loss}) + "\n")
                fh.flush()
                del rot
            print(f"[sweep] {A.name} done", file=sys.stderr, flush=True)
    losses.sort()
    geomean = math.exp(sum(math.log1p(l) for l in losses) / len(losses)) - 1.0      # geometric mean of t_selected / t_best, minus 1
    print(json.dumps({"suite": "sweep", "cells": len(losses), "mean_loss": sum(losses) / len(losses),
                      "geomean_loss": geomean, "median_loss": losses[len(losses) // 2], "max_loss": losses[-1],
                      "file": path}))
    return 0


def run_tiny(args):
    """The tiny configuration (4096^2, Poisson(8) rows, N = 4) is launch-bound: time per call of each
    kernel launched eagerly and replayed from a HIP graph that holds 20 calls."""
    import torch
    from paper_2106_16064_amd import binding as dg
    A, X, label = make_workload("tiny", 4)
    dA = dg.DeviceCsr(A)
    dX = torch.from_numpy(X).cuda()
    dY = torch.empty((A.M, 4), dtype=torch.float32, device="cuda:0")
    out = {}
    per_graph = 20
    side = torch.cuda.Stream()
    for algo in dg.ALGOS:
        name = dg.dgsp_algo_name(algo)
        with torch.cuda.stream(side):
            for _ in range(5):
                dA.spmm(dX, algo=algo, Y=dY)
            side.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                dA.spmm(dX, algo=algo, Y=dY)
            side.synchronize()
            eager = (time.perf_counter() - t0) / args.steps
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(per_graph):
                dA.spmm(dX, algo=algo, Y=dY)
        graph.replay()
        torch.cuda.synchronize()
        reps = max(1, args.steps // per_graph)
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        replay = (time.perf_counter() - t0) / (reps * per_graph)
        out[name] = {"eager_us": eager * 1e6, "graph_us": replay * 1e6}
    sel = dg.dgsp_algo_name(dg.dgsp_select_algo(dA.features, 4))
    print(json.dumps({"suite": "tiny", "workload": label, "nnz": A.nnz, "selected": sel, "per_call": out}))
    return 0


def run_size(args):
    """All four kernels on banded and random matrices of growing size at small N: where the
    second launch of the balanced kernels starts to pay (fits the selector's pr_nnz_max) and where X
    outgrows an L2 (the large-dense-operand rule)."""
    from paper_2106_16064_amd import binding as dg
    from paper_2106_16064_amd import workloads as wl
    os.makedirs(RESULTS_DIR, exist_ok=True)
    path = os.path.join(RESULTS_DIR, args.out or "bench_size.jsonl")
    gens = [(f"stencil27_n{n}", lambda n=n: wl.stencil27_csr(n, seed=0)) for n in (40, 64, 96, 128)]
    gens += [(f"fixed27_M2^{lg}", lambda lg=lg: wl.sweep_csr(1 << lg, 27, "fixed", 0)) for lg in (18, 19, 20, 21)]
    gens += [(f"poisson16_M2^{lg}", lambda lg=lg: wl.sweep_csr(1 << lg, 16, "poisson", 0)) for lg in (18, 20)]
    gens += [(f"{law}{mu}_M2^20", lambda law=law, mu=mu: wl.sweep_csr(1 << 20, mu, law, 0))
             for law, mu in (("fixed", 40), ("fixed", 64), ("poisson", 32))]
    cells = 0
    with open(path, "w") as fh:
        for name, gen in gens:
            A = gen()
            for n in (1, 2, 4, 8):
                rot = Rotation(A, wl.dense_matrix(A.K, n, "uniform", seed=0))
                table = variant_table(rot, args.steps, args.warmup)
                f = rot.mats[0].features
                sel = dg.dgsp_algo_name(dg.dgsp_select_algo(f, n))
                best = min(table, key=table.get)
                fh.write(json.dumps({"matrix": name, "N": n, "M": A.M, "avg_row": f.avg_row, "cv_row": f.cv_row,
                                     "max_row": f.max_row, "nnz": A.nnz, "K": A.K, "col_span": f.col_span, "ms": table, "selected": sel,
                                     "best": best, "loss": table[sel] / table[best] - 1.0}) + "\n")
                fh.flush()
                cells += 1
                del rot
            print(f"[size] {name} done", file=sys.stderr, flush=True)
    print(json.dumps({"suite": "size", "cells": cells, "file": path}))
    return 0


def run_widths(args):
    """The adaptive call over a range of dense widths, multiples of four and not, on three matrix kinds:
    time per call and the kernel the rules picked (what a caller with an odd N gets)."""
    from paper_2106_16064_amd import binding as dg
    from paper_2106_16064_amd import workloads as wl
    os.makedirs(RESULTS_DIR, exist_ok=True)
    path = os.path.join(RESULTS_DIR, args.out or "bench_widths.jsonl")
    widths = list(range(1, 21)) + [24, 31, 32, 33, 40, 41, 47, 48, 63, 64, 65, 96, 100, 128]
    mats = [("R-MAT 2^20, avg degree 16", lambda: wl.rmat_csr(20, 16, seed=0, values="uniform01")),
            ("Poisson(16) rows, 2^18 rows", lambda: wl.sweep_csr(1 << 18, 16, "poisson", 0)),
            ("27-point stencil 64^3", lambda: wl.stencil27_csr(64, seed=0))]
    cells = 0
    pad = args.ld_multiple
    with open(path, "w") as fh:
        for label, gen in mats:
            A = gen()
            for n in widths:
                rot = Rotation(A, wl.dense_matrix(A.K, n, "uniform", seed=0))
                if pad:
                    # rows of X and Y padded to a multiple of `pad` floats and passed as views: what the library
                    # recommends to callers with odd widths (rows then start on line boundaries)
                    import torch
                    ld = -(-n // pad) * pad
                    Xp = [torch.zeros((A.K, ld), dtype=torch.float32, device="cuda:0") for _ in range(rot.copies)]
                    Yp = [torch.empty((A.M, ld), dtype=torch.float32, device="cuda:0") for _ in range(rot.copies)]
                    for j in range(rot.copies):
                        Xp[j][:, :n] = rot.X[j]

                    def call(i):
                        j = i % rot.copies
                        m = rot.mats[j]
                        dg.dgsp_spmm_csr_ld(m.M, m.K, n, m.nnz, m.rowptr, m.colidx, m.vals, Xp[j][:, :n], Yp[j][:, :n],
                                            dg.AUTO, m.features)
                else:
                    def call(i):
                        rot.step(i, dg.AUTO)
                us = median(time_events(None, call, max(5, min(args.steps, 30)), 3)) * 1e3
                sel = dg.dgsp_algo_name(dg.dgsp_select_algo(rot.mats[0].features, n))
                fh.write(json.dumps({"matrix": label, "N": n, "nnz": A.nnz, "us": us, "selected": sel,
                                     "ld": (-(-n // pad) * pad) if pad else n}) + "\n")
                fh.flush()
                cells += 1
                del rot
            print(f"[widths] {label} done", file=sys.stderr, flush=True)
    print(json.dumps({"suite": "widths", "cells": cells, "file": path}))
    return 0


def run_ablation(args):
    """Each optimisation of Section 2.1 against the kernel without it, on a grid of 27 R-MAT matrices
    (3 sizes x 3 densities x 3 skews; the paper's own 27 parameter sets are not published):
    N = 1: all four kernels and the balanced kernel with a serial segment scan (which design point wins how
    often; Section 2.1.1); N = 2: vector-type dense-row loads
    against scalar loads = two passes (Section 2.1.2); N = 128: LDS-staged sparse rows against none
    (Section 2.1.3)."""
    from paper_2106_16064_amd import binding as dg
    from paper_2106_16064_amd import workloads as wl
    os.makedirs(RESULTS_DIR, exist_ok=True)
    path = os.path.join(RESULTS_DIR, args.out or "bench_ablation.jsonl")
    skews = RMAT_GRID_SKEWS
    k = max(5, min(args.steps, 20))

    def med(fn):
        return median(time_events(None, fn, k, 3))

    rows = []
    with open(path, "w") as fh:
        for scale in (16, 18, 20):
            for deg in (4, 16, 32):
                for sname, abcd in skews.items():
                    A = wl.rmat_csr(scale, deg, abcd, seed=0, values="uniform01")
                    row = {"matrix": f"rmat_s{scale}_d{deg}_{sname}", "nnz": A.nnz, "stats": A.stats()}
                    rot = Rotation(A, wl.dense_matrix(A.K, 1, "uniform", seed=0))
                    row["spmv_ms"] = variant_table(rot, k, 3)
                    # the third alternative of Section 2.1.1: balanced, segment reduction as a serial scan
                    row["spmv_ms"]["nb_pr_serial_scan"] = med(lambda i: rot.ablation(i, dg.NB_PR, dg.ABL_SERIAL_SEGMENT_SCAN))
                    row["spmv_ms"]["nb_pr_item_tiles"] = med(lambda i: rot.ablation(i, dg.NB_PR, dg.ABL_ITEM_TILES))
                    row["spmv_ms"]["nb_pr_entry_blocks"] = med(lambda i: rot.ablation(i, dg.NB_PR, dg.ABL_ENTRY_BLOCKS))
                    # the textbook kernel: one lane per row, entries read straight from memory (no staging, no balancing)
                    row["spmv_ms"]["csr_scalar"] = med(lambda i: rot.ablation(i, dg.RS_SR, dg.ABL_NO_SPARSE_STAGING))
                    del rot
                    rot = Rotation(A, wl.dense_matrix(A.K, 2, "uniform", seed=0))
                    row["n2_ms"] = {}
                    for algo in (dg.RS_PR, dg.NB_PR):
                        nm = dg.dgsp_algo_name(algo)
                        row["n2_ms"][nm] = med(lambda i: rot.ablation(i, algo, 0))
                        row["n2_ms"][nm + "_scalar_loads"] = med(lambda i: rot.ablation(i, algo, dg.ABL_SCALAR_DENSE_LOADS))
                    del rot
                    rot = Rotation(A, wl.dense_matrix(A.K, 128, "uniform", seed=0), copies=2)
                    row["n128_ms"] = {
                        "rs_sr": med(lambda i: rot.ablation(i, dg.RS_SR, 0)),
                        "rs_sr_no_staging": med(lambda i: rot.ablation(i, dg.RS_SR, dg.ABL_NO_SPARSE_STAGING)),
                        "nb_sr": med(lambda i: rot.ablation(i, dg.NB_SR, 0))}
                    del rot
                    rows.append(row)
                    fh.write(json.dumps(row) + "\n")
                    fh.flush()
                    print(f"[ablation] {row['matrix']} done", file=sys.stderr, flush=True)

    def geomean(v):
        return float(np.exp(np.mean(np.log(v))))

    wins, design = {}, {}
    points = ("rs_sr", "rs_pr", "nb_pr_serial_scan", "nb_pr")     # Section 2.1.1: baseline, parallel only, balance only, both
    for r in rows:
        four = {k: r["spmv_ms"][k] for k in ("rs_sr", "rs_pr", "nb_sr", "nb_pr")}
        b = min(four, key=four.get)
        wins[b] = wins.get(b, 0) + 1
        d = min(points, key=lambda k: r["spmv_ms"][k if k != "nb_pr" else "nb_pr_entry_blocks"])
        design[d] = design.get(d, 0) + 1
    print(json.dumps({
        "suite": "ablation", "matrices": len(rows), "file": path,
        "spmv_best_kernel_counts": wins,
        "spmv_design_points_best_counts": design,
        "segment_scan_dpp_vs_serial_speedup_N1": geomean([r["spmv_ms"]["nb_pr_serial_scan"] / r["spmv_ms"]["nb_pr_entry_blocks"] for r in rows]),
        "entry_blocks_vs_item_tiles_speedup_N1": geomean([r["spmv_ms"]["nb_pr_item_tiles"] / r["spmv_ms"]["nb_pr_entry_blocks"] for r in rows]),
        "entry_blocks_vs_item_tiles_speedup_N1_from_6M_entries": geomean(
            [r["spmv_ms"]["nb_pr_item_tiles"] / r["spmv_ms"]["nb_pr_entry_blocks"] for r in rows if r["nnz"] >= 6e6] or [1.0]),
        "vector_dense_loads_speedup_N2": {a: geomean([r["n2_ms"][a + "_scalar_loads"] / r["n2_ms"][a] for r in rows])
                                          for a in ("rs_pr", "nb_pr")},
        "best_of_four_vs_csr_scalar_speedup_N1": geomean([r["spmv_ms"]["csr_scalar"] / min(r["spmv_ms"][k] for k in ("rs_sr", "rs_pr", "nb_sr", "nb_pr")) for r in rows]),
        "sparse_staging_speedup_N128": geomean([r["n128_ms"]["rs_sr_no_staging"] / r["n128_ms"]["rs_sr"] for r in rows])}))
    return 0


def run_layouts(args):
    """The wide-N layouts of the balanced sequential kernel on the GNN-style configuration (R-MAT 2^20, row-normalised,
    N = 64, 128 and 256) and on a matrix with uniform columns: column blocks of 64 (what ships) or 32, tied to XCDs
    (what ships from N = 128 on) or not; whole call, event-timed, for the comparison table under profiles/."""
    from paper_2106_16064_amd import binding as dg
    from paper_2106_16064_amd import workloads as wl
    os.makedirs(RESULTS_DIR, exist_ok=True)
    path = os.path.join(RESULTS_DIR, args.out or "bench_layouts.jsonl")
    variants = {"blocks_of_64_on_xcds (ships at N >= 128)": 0, "blocks_of_64_any_xcd": dg.ABL_BLOCKS_OFF_XCDS,
                "blocks_of_32_on_xcds": dg.ABL_COLUMN_BLOCKS_32,
                "blocks_of_32_any_xcd": dg.ABL_COLUMN_BLOCKS_32 | dg.ABL_BLOCKS_OFF_XCDS}
    cells = 0
    with open(path, "w") as fh:
        for name in ("rmat_gnn", "uniform64"):
            for n in (64, 128, 256):
                A, X, label = make_workload(name, n)
                rot = Rotation(A, X)
                rec = {"workload": label, "N": n, "nnz": A.nnz, "algorithmic_bytes": algorithmic_bytes(A, n), "us": {}}
                for vname, sw in variants.items():
                    ms = time_events(None, lambda i: rot.ablation(i, dg.NB_SR, sw), max(8, min(args.steps, 20)), 3)
                    rec["us"][vname] = median(ms) * 1e3
                fh.write(json.dumps(rec) + "\n")
                fh.flush()
                cells += 1
                print(f"[layouts] {label}: " + ", ".join(f"{k} {v:.0f} us" for k, v in rec["us"].items()), file=sys.stderr, flush=True)
                del rot
    print(json.dumps({"suite": "layouts", "cells": cells, "file": path}))
    return 0


def run_gather(args):
    """dgsp_gather_probe on synthetic index patterns (55.7 M indices into 2 M floats, the stencil's sizes): what the
    memory pipeline charges for a gather as a function of how the lanes of a wave fall onto 128-byte lines."""
    import torch
    from paper_2106_16064_amd import binding as dg
    os.makedirs(RESULTS_DIR, exist_ok=True)
    path = os.path.join(RESULTS_DIR, args.out or "bench_gather.jsonl")
    n, K = 55742968, 2097152
    out = torch.empty(dg.dgsp_gather_probe_out_len(), device="cuda:0")
    x = torch.zeros(K, device="cuda:0")
    i = torch.arange(n, device="cuda:0", dtype=torch.int64)
    patterns = {
        "consecutive (every wave one run of 64)": lambda: i % K,
        "runs of 16 consecutive at scattered places": lambda: (i // 16) * 977 % (K - 16) + (i % 16),
        "runs of 4 consecutive at scattered places": lambda: (i // 4) * 977 % (K - 4) + (i % 4),
        "runs of 3 consecutive at scattered places": lambda: (i // 3) * 977 % (K - 4) + (i % 3),
        "stride 977 (every lane its own line)": lambda: (i * 977) % K,
        "all lanes the same element": lambda: torch.zeros_like(i),
    }
    A, _, _ = make_workload("stencil", 1)
    patterns["the 27-point stencil's own column indices"] = lambda: torch.from_numpy(A.colidx).to("cuda:0").to(torch.int64)
    rows = []
    with open(path, "w") as fh:
        for name, make in patterns.items():
            idx = make().to(torch.int32)
            ms = time_events(None, lambda k: dg.dgsp_gather_probe(out, x, idx), max(8, min(args.steps, 20)), 3)
            rec = {"pattern": name, "indices": int(idx.numel()), "us": median(ms) * 1e3}
            rows.append(rec)
            fh.write(json.dumps(rec) + "\n")
            print(f"[gather] {name}: {rec['us']:.1f} us", file=sys.stderr, flush=True)
            del idx
    print(json.dumps({"suite": "gather", "cells": len(rows), "file": path}))
    return 0


def run_colranges(args):
    """What passes over column ranges would do to the GNN-style configuration (R-MAT 2^20, N = 128): A is cut on the
    host into P matrices that hold the entries of one range of columns each (all M rows, CSR order kept), and
    Y = A_0 X, then Y += A_p X for the others, through the library's own calls (the scaled form with beta = 1).
    Every pass then touches 1/P of the rows of X - and reads and writes all of Y again."""
    import numpy as np
    import torch
    from paper_2106_16064_amd import binding as dg
    from paper_2106_16064_amd import workloads as wl
    os.makedirs(RESULTS_DIR, exist_ok=True)
    path = os.path.join(RESULTS_DIR, args.out or "bench_colranges.jsonl")
    n = args.n or 128
    A, X, label = make_workload(args.workload or "rmat_gnn", n)
    Xd = torch.from_numpy(X).to("cuda:0")
    Y = torch.empty((A.M, n), dtype=torch.float32, device="cuda:0")
    row_of = np.repeat(np.arange(A.M, dtype=np.int64), A.row_lengths())
    steps = max(6, min(args.steps, 12))
    with open(path, "w") as fh:
        for how in ("equal_width", "equal_entries"):
            for P in (1, 2, 4, 8, 16):
                if how == "equal_width":
                    cuts = [A.K * q // P for q in range(P + 1)]
                else:
                    srt = np.sort(A.colidx)
                    cuts = [0] + [int(srt[A.nnz * q // P]) for q in range(1, P)] + [A.K]
                parts = []
                for q in range(P):
                    keep = (A.colidx >= cuts[q]) & (A.colidx < cuts[q + 1])
                    counts = np.bincount(row_of[keep], minlength=A.M)
                    rowptr = np.concatenate(([0], np.cumsum(counts))).astype(np.int32)
                    parts.append(dg.DeviceCsr(wl.CsrMatrix(A.M, A.K, rowptr, A.colidx[keep], A.vals[keep], f"{label} cols {q}/{P}")))

                def call(_):
                    for q, m in enumerate(parts):
                        if q == 0:
                            m.spmm(Xd, algo=dg.AUTO, Y=Y)
                        else:
                            dg.dgsp_spmm_csr_axpby(m.M, m.K, n, m.nnz, m.rowptr, m.colidx, m.vals, Xd, Y, 1.0, 1.0, dg.AUTO, m.features)
                ms = time_events(None, call, steps, 2)
                rec = {"workload": label, "N": n, "cut": how, "passes": P, "entries_per_pass": [int(m.nnz) for m in parts],
                       "kernels": [dg.dgsp_algo_name(dg.dgsp_select_algo(m.features, n)) for m in parts], "us": median(ms) * 1e3}
                fh.write(json.dumps(rec) + "\n")
                fh.flush()
                print(f"[colranges] {how} P={P}: {rec['us']:.0f} us", file=sys.stderr, flush=True)
                del parts
                torch.cuda.empty_cache()
    print(json.dumps({"suite": "colranges", "file": path}))
    return 0


RMAT_GRID_SKEWS = {"powerlaw": (0.57, 0.19, 0.19, 0.05), "mild": (0.45, 0.15, 0.15, 0.25), "uniform": (0.25, 0.25, 0.25, 0.25)}


def run_holdout(args):
    """Scores the shipped selection rules on inputs they were not fitted on: the 27-matrix R-MAT grid of the
    ablation suite (3 sizes x 3 densities x 3 skews) and seven further row-length laws at 2^18 rows
    (workloads.HOLDOUT_LAWS), each at N in {1, 4, 8, 32, 128}; all four kernels timed per cell, loss of the rules'
    choice against the fastest.  Reports mean, worst and the cells above 10 %."""
    from paper_2106_16064_amd import binding as dg
    from paper_2106_16064_amd import workloads as wl
    os.makedirs(RESULTS_DIR, exist_ok=True)
    path = os.path.join(RESULTS_DIR, args.out or "bench_holdout.jsonl")
    gens = [(f"rmat_s{scale}_d{deg}_{sname}", lambda scale=scale, deg=deg, abcd=abcd: wl.rmat_csr(scale, deg, abcd, seed=0, values="uniform01"))
            for scale in (16, 18, 20) for deg in (4, 16, 32) for sname, abcd in RMAT_GRID_SKEWS.items()]
    gens += [(f"law_{law}", lambda law=law: wl.holdout_law_csr(law, 1 << 18, seed=0)) for law in wl.HOLDOUT_LAWS]
    if args.workload:
        gens = [g for g in gens if g[0].startswith(args.workload)]
    k = max(5, min(args.steps, 10))
    cells = []
    with open(path, "w") as fh:
        for name, gen in gens:
            A = gen()
            for n in (1, 4, 8, 32, 128):
                rot = Rotation(A, wl.dense_matrix(A.K, n, "uniform", seed=0), copies=2 if A.nnz * n > 3e8 else None)
                table = variant_table(rot, k, 2)
                f = rot.mats[0].features
                sel = dg.dgsp_algo_name(dg.dgsp_select_algo(f, n))
                best = min(table, key=table.get)
                rec = {"matrix": name, "N": n, "M": A.M, "avg_row": f.avg_row, "cv_row": f.cv_row, "max_row": f.max_row, "nnz": A.nnz,
                       "K": A.K, "col_span": f.col_span, "ms": table, "selected": sel, "best": best,
                       "loss": table[sel] / table[best] - 1.0}
                cells.append(rec)
                fh.write(json.dumps(rec) + "\n")
                fh.flush()
                del rot
            print(f"[holdout] {name} done", file=sys.stderr, flush=True)
    losses = [c["loss"] for c in cells]
    over = [c for c in cells if c["loss"] > 0.10]
    print(json.dumps({"suite": "holdout", "cells": len(cells), "file": path, "mean_loss": sum(losses) / len(losses),
                      "worst_loss": max(losses), "cells_over_10pct": len(over),
                      "over_10pct": [{"matrix": c["matrix"], "N": c["N"], "selected": c["selected"], "best": c["best"],
                                      "loss": round(c["loss"], 3)} for c in over]}))
    return 0


THRESHOLD_NAMES = ("n_parallel_max", "pr_avg_row_min", "pr_cv_max", "sr_cv_min", "sr_stdv_min", "pr_nnz_max",
                   "short_avg_row_max", "short_max_row_max", "wide_parallel_n", "big_x_bytes_min", "big_x_cv_max",
                   "big_x_avg_row_max", "short_min_waves", "pr_small_nnz_max", "pr_small_cv_max")


def sr_lanes(N):
    """Lanes per row of the sequential kernels at width N (a power of two covering N in lanes of four columns)."""
    if N < 4:
        return 1
    g = 1
    while g < (N + 3) // 4:
        g *= 2
    return min(g, 64)


def rules_choose(r, t):
    """The library's selection rules (dgsp_select_algo) on a bench record r with thresholds t (a dict)."""
    N = r["N"]
    M = r.get("M") or (round(r["nnz"] / r["avg_row"]) if r["avg_row"] > 0 else 0)
    if (r["nnz"] > 0 and r["avg_row"] <= t["short_avg_row_max"] and r["max_row"] <= t["short_max_row_max"]
            and M * sr_lanes(N) >= 64 * t["short_min_waves"]):
        return "rs_sr"
    if N <= t["n_parallel_max"]:
        if (t["big_x_bytes_min"] > 0 and r.get("K", 0) * N * 4 >= t["big_x_bytes_min"] and r["cv_row"] <= t["big_x_cv_max"]
                and r["avg_row"] <= t["big_x_avg_row_max"] and r.get("col_span", 0.0) >= 0.5):
            return "rs_sr"
        if 0 < r["nnz"] <= t["pr_small_nnz_max"] and r["cv_row"] <= t["pr_small_cv_max"]:
            return "rs_pr"
        row_split = r["avg_row"] >= t["pr_avg_row_min"] and r["cv_row"] <= t["pr_cv_max"] and r["nnz"] < t["pr_nnz_max"]
        return "rs_pr" if row_split else "nb_pr"
    if not (r["cv_row"] > t["sr_cv_min"] and r["avg_row"] * r["cv_row"] > t["sr_stdv_min"]):
        return "rs_sr"
    return "nb_pr" if N <= t["wide_parallel_n"] else "nb_sr"


def run_fit(args):
    """Grid-fits the selector thresholds.  Data: the seed-0 matrices of a finished sweep
    (bench_sweep.jsonl under RESULTS_DIR) plus, if that suite ran, the larger matrices of
    bench_size.jsonl (the sweep alone cannot place the size guards); checked on the
    seed-1 matrices of the sweep and, if that suite ran, scored on bench_holdout.jsonl.  No GPU needed."""
    path = args.out or os.path.join(RESULTS_DIR, "bench_sweep.jsonl")
    rows = [json.loads(l) for l in open(path)]
    here = os.path.dirname(path) or "."

    def load(name):
        f = os.path.join(here, name)
        return [json.loads(l) for l in open(f)] if os.path.exists(f) else []

    big, hold = load("bench_size.jsonl"), load("bench_holdout.jsonl")
    inf = float("inf")
    off = dict(pr_nnz_max=inf, short_avg_row_max=0.0, short_max_row_max=0, wide_parallel_n=0, big_x_bytes_min=0,
               big_x_cv_max=0.0, big_x_avg_row_max=0.0, short_min_waves=0, pr_small_nnz_max=0, pr_small_cv_max=0.0)

    def losses(rs, t):
        return [r["ms"][rules_choose(r, t)] / min(r["ms"].values()) - 1 for r in rs]

    def loss(rs, t):
        l = losses(rs, t)
        return (sum(l) / len(l), max(l)) if l else (0.0, 0.0)

    fit = [r for r in rows if r["matrix"].endswith("_s0")]
    test = [r for r in rows if r["matrix"].endswith("_s1")]
    train = fit + big

    # stage 1: the paper's tree (5 thresholds), added rules off; stage 2: the added rules on the 20 best trees
    tree = [dict(off, n_parallel_max=npm, pr_avg_row_min=a, pr_cv_max=c, sr_cv_min=sc, sr_stdv_min=ss)
            for npm in (1, 2, 4, 8) for a in (0, 2, 8, 12, 24, 48, 1e9)
            for c in (0.05, 0.1, 0.2, 0.3, 0.5, 1.0, 2.0, 4.0, 1e30) for sc in (0.3, 0.8, 1.0, 1.5, 2.0, 3.5, 1e9)
            for ss in (0, 3, 10, 30, 60)]
    ranked = sorted(tree, key=lambda t: loss(train, t)[0])
    added = [dict(pr_nnz_max=nm, short_avg_row_max=a, short_max_row_max=m, wide_parallel_n=w)
             for nm in (5e6, 1e7, 2e7, 4e7, inf)
             for (a, m) in [(0.0, 0)] + [(a, m) for a in (5, 10, 20, 40) for m in (16, 32, 64, 128, 512)] for w in (0, 8)]
    best = min((dict(t, **x) for t in ranked[:20] for x in added), key=lambda t: loss(train, t)[0])
    # stage 3: the large-dense-operand rule; stage 4: the row-count condition of the short-row rule and the
    # small-matrix rule of the parallel side
    bigx = [dict()] + [dict(big_x_bytes_min=b, big_x_cv_max=c, big_x_avg_row_max=a)
                       for b in (4.2e6, 6e6, 1.2e7) for c in (0.05, 0.2, 0.3) for a in (48, 64, 128)]
    best = min((dict(best, **x) for x in bigx), key=lambda t: loss(train, t)[0])
    small = [dict(short_min_waves=w, pr_small_nnz_max=n, pr_small_cv_max=c)
             for w in (0, 1024, 2048, 4096) for n in (0, 2e6, 4e6, 8e6) for c in (0.15, 0.3, 0.6)]
    best = min((dict(best, **x) for x in small), key=lambda t: loss(train, t)[0])
    grid_best = best
    # what is reported below is what ships: the library's defaults (the grid's optimum beside them; the loss is
    # flat in several thresholds, so the two differ without one being better)
    try:
        from paper_2106_16064_amd import binding as dg
        d = dg.dgsp_get_thresholds()
        best = {k: getattr(d, k) for k in THRESHOLD_NAMES}
        shipped = True
    except Exception:            # no library built: report the grid's optimum
        shipped = False
    paper = min((t for t in tree if t["n_parallel_max"] == 4 and t["pr_cv_max"] == 1e30 and t["sr_stdv_min"] == 0),
                key=lambda t: loss(fit, t)[0])
    single = {k: (sum(r["ms"][k] / min(r["ms"].values()) - 1 for r in rows) / len(rows)) for k in rows[0]["ms"]}
    per_n = {}
    for r, l in zip(rows, losses(rows, best)):
        per_n.setdefault(r["N"], []).append(l)

    def variant(**kw):            # the shipped thresholds with some of the added rules switched off
        t = dict(best, **kw)
        return {"sweep_fit": loss(fit, t)[0], "sweep_heldout": loss(test, t)[0], "size_cells": loss(big, t)[0],
                "holdout_cells": loss(hold, t)[0]}

    def over(rs, t, limit=0.10):
        return [{"matrix": r["matrix"], "N": r["N"], "selected": rules_choose(r, t), "best": min(r["ms"], key=r["ms"].get),
                 "loss": round(l, 3)} for r, l in zip(rs, losses(rs, t)) if l > limit]

    print(json.dumps({
        "suite": "fit", "sweep_cells": len(rows), "size_cells": len(big), "holdout_cells": len(hold),
        "thresholds": best, "thresholds_are_library_defaults": shipped,
        "grid_fit": {"thresholds": grid_best, "sweep_fit": loss(fit, grid_best)[0],
                     "sweep_heldout": loss(test, grid_best)[0], "size_cells": loss(big, grid_best)[0]},
        "mean_loss_fit_seed0": loss(fit, best)[0], "mean_loss_heldout_seed1": loss(test, best)[0],
        "mean_loss_sweep_all": loss(rows, best)[0], "max_loss_sweep_all": loss(rows, best)[1],
        "geomean_loss_sweep_all": math.exp(sum(math.log1p(l) for l in losses(rows, best)) / len(rows)) - 1.0,
        "mean_loss_size_cells": loss(big, best)[0], "max_loss_size_cells": loss(big, best)[1],
        "holdout": {"mean_loss": loss(hold, best)[0], "worst_loss": loss(hold, best)[1],
                    "cells_over_10pct": len(over(hold, best)), "over_10pct": over(hold, best)},
        "over_10pct_sweep": over(rows, best), "over_10pct_size": over(big, best),
        "added_rules_off": {"no_short_row_rule": variant(short_avg_row_max=0.0, short_max_row_max=0),
                            "short_rows_at_any_row_count": variant(short_min_waves=0),
                            "no_small_matrix_rule": variant(pr_small_nnz_max=0),
                            "no_size_guard": variant(pr_nnz_max=inf),
                            "no_eight_column_rule": variant(wide_parallel_n=0),
                            "no_large_x_rule": variant(big_x_bytes_min=0),
                            "none": variant(**off)},
        "paper_shaped_tree": {"thresholds": paper, "mean_loss_fit": loss(fit, paper)[0],
                              "mean_loss_heldout": loss(test, paper)[0], "mean_loss_size_cells": loss(big, paper)[0],
                              "mean_loss_holdout_cells": loss(hold, paper)[0]},
        "always_one_kernel_mean_loss": single,
        "mean_loss_per_N": {str(n): sum(v) / len(v) for n, v in sorted(per_n.items())}}))
    return 0


def run_kernel(args):
    """One kernel in a plain loop, for rocprofv3."""
    import torch
    from paper_2106_16064_amd import binding as dg
    A, X, label = make_workload(args.workload or "rmat_spmv", args.n or 1)
    rot = Rotation(A, X, copies=1 if args.warm else None)
    algo = {"rs_sr": 0, "rs_pr": 1, "nb_sr": 2, "nb_pr": 3, "auto": -1}[args.algo]
    ms = time_steps(rot, algo, args.steps, args.warmup, warm=args.warm)
    if args.copy_calibration:
        n = 1 << 28
        src = torch.zeros(n, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dg.dgsp_copy_f32(dst, src, n)
        torch.cuda.synchronize()
    print(json.dumps({"suite": "kernel", "workload": label, "algo": args.algo, "ms_per_step": ms,
                      "algorithmic_bytes": algorithmic_bytes(A, X.shape[1]),
                      "no_reuse_bytes": 8 * A.nnz + 4 * A.nnz * X.shape[1] + 4 * A.M * X.shape[1], "copies": rot.copies}))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--suite", default="headline", choices=["headline", "configs", "sweep", "size", "ablation", "tiny", "kernel", "fit", "widths", "holdout", "layouts", "gather", "colranges"])
    ap.add_argument("--workload", default=None)
    ap.add_argument("--n", type=int, default=None)
    ap.add_argument("--algo", default="auto")
    ap.add_argument("--warm", action="store_true", help="kernel suite: reuse one buffer set (cache-warm)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="kernel suite: also run five 1 GiB dgsp_copy_f32 launches (byte-counter calibration)")
    ap.add_argument("--no-cells", action="store_true", help="default suite: only the headline workload, no further cells")
    ap.add_argument("--ld-multiple", type=int, default=0,
                    help="widths suite: pad the rows of X and Y to a multiple of this many floats and pass views")
    ap.add_argument("--sweep-m", type=int, default=1 << 18)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    if args.suite == "fit":
        return run_fit(args)
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (one MI355X); run with --gpus 1", file=sys.stderr)
        return 2
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU fallback", file=sys.stderr)
        return 2
    from paper_2106_16064_amd import binding as dg
    dg.lib()
    return {"headline": run_headline, "configs": run_configs, "sweep": run_sweep, "size": run_size,
            "ablation": run_ablation, "tiny": run_tiny, "kernel": run_kernel, "widths": run_widths,
            "holdout": run_holdout, "layouts": run_layouts, "gather": run_gather, "colranges": run_colranges}[args.suite](args)


if __name__ == "__main__":
    sys.exit(main())
