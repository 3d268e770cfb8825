"""CPU oracle for the CSR SpMV/SpMM hot path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the HIP library:
no headers, helpers, tables or pre/post-processing, and it never imports the
GPU package.

Contents
--------
``spmm_ref``        fp64 triple loop in C (``spmm_ref.c``), the definition of
                    ``Y = A X`` from the paper's problem statement (Section 1).
``spmm_ref_loops``  the same definition as pure-Python loops, for tiny inputs;
                    it exists so that the C build itself has a second opinion.
``row_features``    mean and standard deviation of the CSR row lengths, the
                    two statistics the paper's selection rules use
                    (Section 2.2: ``avg_row`` and ``stdv_row``).
``within_bound``    the acceptance test ``|Y - Yref| <= tol * (|A| |X|)``.

Parity status: ``spmm_ref`` / ``spmm_ref_loops`` are pinned by
``tests/test_oracle.py`` (dense matmul, an independent sparse library, brute
force over COO triples, algebraic invariants and closed forms on the benchmark
generators).  ``row_features`` is pinned by closed forms.  The paper prints no
worked numeric example, so there is no printed value to compare with.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "spmm_ref.c"
_LIB = _HERE / "liboracle_spmm.so"
_lib = None


def build(force: bool = False) -> Path:
    """Compile ``spmm_ref.c`` with gcc into ``liboracle_spmm.so`` (in place)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
               "-ffp-contract=off", "-o", str(_LIB), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_LIB))
        lib.oracle_spmm_csr.restype = ctypes.c_int
        lib.oracle_spmm_csr.argtypes = [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    """Threads the C oracle uses when ``nthreads`` is left at 0."""
    return int(_load().oracle_max_threads())


def _as(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def spmm_ref(M, K, N, rowptr, colidx, vals, X, *, with_bound=True, nthreads=0):
    """Yref (and the bound |A||X|) as fp64 arrays of shape (M, N).

    Paper Section 1: ``Y[M x N] = A[M x K] X[K x N]``; fp32 inputs, every
    product and sum in fp64, stored entries taken in CSR order.
    """
    rowptr = _as(rowptr, np.int32)
    colidx = _as(colidx, np.int32)
    vals = _as(vals, np.float32)
    X = _as(X, np.float32).reshape(K, N) if K * N else np.zeros((K, N), np.float32)
    if rowptr.shape != (M + 1,) or colidx.shape != vals.shape:
        raise ValueError("rowptr must hold M+1 entries; colidx and vals must have equal length")
    if colidx.size < int(rowptr.max(initial=0)):
        raise ValueError("colidx/vals shorter than the largest rowptr entry")
    yref = np.empty((M, N), dtype=np.float64)
    bnd = np.empty((M, N), dtype=np.float64) if with_bound else None
    rc = _load().oracle_spmm_csr(
        M, K, N, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data,
        X.ctypes.data, yref.ctypes.data,
        bnd.ctypes.data if with_bound else None, int(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_spmm_csr rejected the matrix (code {rc})")
    return (yref, bnd) if with_bound else yref


def spmm_ref_loops(M, K, N, rowptr, colidx, vals, X):
    """Same definition as :func:`spmm_ref`, three Python loops (tiny inputs)."""
    X = np.asarray(X, dtype=np.float32).reshape(K, N)
    yref = np.zeros((M, N), dtype=np.float64)
    bnd = np.zeros((M, N), dtype=np.float64)
    for i in range(M):
        for p in range(int(rowptr[i]), int(rowptr[i + 1])):
            a = float(vals[p])
            k = int(colidx[p])
            for n in range(N):
                x = float(X[k, n])
                yref[i, n] += a * x
                bnd[i, n] += abs(a) * abs(x)
    return yref, bnd


def row_features(rowptr):
    """Row-length statistics used by the selection rules (paper Section 2.2).

    ``avg_row`` is the mean and ``stdv_row`` the population standard deviation
    of ``rowptr[i+1]-rowptr[i]`` over all M rows, empty rows included (the
    paper does not say population or sample; with M in the millions the two
    agree to six digits).  Returned as a dict of Python floats/ints.
    """
    rowptr = np.asarray(rowptr, dtype=np.int64)
    lens = np.diff(rowptr)
    M = int(lens.size)
    if M == 0:
        return dict(M=0, nnz=0, avg_row=0.0, stdv_row=0.0, max_row=0, min_row=0)
    avg = float(lens.sum()) / M
    var = float(((lens.astype(np.float64) - avg) ** 2).sum()) / M
    return dict(M=M, nnz=int(rowptr[-1]), avg_row=avg, stdv_row=float(np.sqrt(var)),
                max_row=int(lens.max()), min_row=int(lens.min()))


def within_bound(Y, yref, bnd, tol=1e-5):
    """Elementwise acceptance test ``|Y - Yref| <= tol * bnd``.

    Returns ``(ok, worst)`` where ``worst`` is the largest ratio
    ``|Y - Yref| / bnd`` over entries with ``bnd > 0`` (0 if none); entries
    with ``bnd == 0`` (empty rows, all-zero products) must equal exactly 0.
    """
    Y = np.asarray(Y, dtype=np.float64).reshape(yref.shape)
    err = np.abs(Y - yref)
    ok = bool(np.all(err <= tol * bnd))
    pos = bnd > 0
    worst = float((err[pos] / bnd[pos]).max()) if pos.any() else 0.0
    return ok, worst
