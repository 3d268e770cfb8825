"""Thin ctypes binding over ``libdgsp.so`` with the same names as the C-ABI
(``include/dgsp.h``).  Argument marshalling only: every step of the
multiplication runs inside the HIP library.  Tensors are ``torch`` CUDA(HIP)
tensors used purely as device memory; the stream is torch's current stream.

There is no CPU fallback: if the shared library has not been built the first
call raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

RS_SR, RS_PR, NB_SR, NB_PR, AUTO = 0, 1, 2, 3, -1
ALGOS = (RS_SR, RS_PR, NB_SR, NB_PR)
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_LAUNCH = 0, 1, 2, 3

LIB_PATH = Path(__file__).resolve().parent / "libdgsp.so"

EXPORTS = (
    "dgsp_spmm_csr", "dgsp_spmm_csr_nnz", "dgsp_spmm_csr_auto", "dgsp_select_algo",
    "dgsp_get_thresholds", "dgsp_set_thresholds", "dgsp_features_from_rowptr_host",
    "dgsp_copy_f32", "dgsp_algo_name", "dgsp_status_string",
    "dgsp_spmm_csr_phase", "dgsp_gather_probe", "dgsp_gather_probe_out_len", "dgsp_features_from_csr_host",
    "dgsp_spmm_csr_ablation", "dgsp_features_from_csr_device", "dgsp_autotune",
    "dgsp_spmm_csr_ld", "dgsp_spmm_csr_axpby", "dgsp_features_from_csr_device_noalloc",
    "dgsp_floor_probe", "dgsp_floor_probe_out_len", "dgsp_spmm_csr_i64", "dgsp_spmm_csr_i64_workspace_bytes",
)
PHASE_ALL, PHASE_PREPARE, PHASE_MAIN = 0, 1, 2
ABL_SCALAR_DENSE_LOADS, ABL_NO_SPARSE_STAGING, ABL_ITEM_TILES, ABL_SERIAL_SEGMENT_SCAN = 1, 2, 4, 8
ABL_COLUMN_BLOCKS_32, ABL_BLOCKS_OFF_XCDS, ABL_ENTRY_BLOCKS = 16, 32, 64
FEATURES_WORKSPACE_BYTES = 64
PROBE_GATHER, PROBE_STREAM_GATHER_FMA, PROBE_ROW_GATHER = 0, 1, 2


class Features(ctypes.Structure):
    """``dgsp_features_t``"""
    _fields_ = [("M", ctypes.c_int64), ("K", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("avg_row", ctypes.c_double), ("stdv_row", ctypes.c_double), ("cv_row", ctypes.c_double),
                ("max_row", ctypes.c_int64), ("min_row", ctypes.c_int64), ("col_span", ctypes.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class Thresholds(ctypes.Structure):
    """``dgsp_thresholds_t``"""
    _fields_ = [("n_parallel_max", ctypes.c_int64), ("pr_avg_row_min", ctypes.c_double),
                ("pr_cv_max", ctypes.c_double), ("sr_cv_min", ctypes.c_double),
                ("sr_stdv_min", ctypes.c_double), ("pr_nnz_max", ctypes.c_int64),
                ("short_avg_row_max", ctypes.c_double), ("short_max_row_max", ctypes.c_int64),
                ("wide_parallel_n", ctypes.c_int64), ("big_x_bytes_min", ctypes.c_int64),
                ("big_x_cv_max", ctypes.c_double), ("big_x_avg_row_max", ctypes.c_double),
                ("short_min_waves", ctypes.c_int64), ("pr_small_nnz_max", ctypes.c_int64),
                ("pr_small_cv_max", ctypes.c_double)]


class DgspError(RuntimeError):
    pass


_lib = None


def lib():
    """The loaded library (raises if it is missing: build it first with
    ``python -m paper_2106_16064_amd.build``)."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise DgspError(f"{LIB_PATH} is missing: run `python -m paper_2106_16064_amd.build` "
                            "(there is no CPU fallback)")
        L = ctypes.CDLL(str(LIB_PATH))
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        L.dgsp_spmm_csr.restype = ci
        L.dgsp_spmm_csr.argtypes = [i64, i64, i64, vp, vp, vp, vp, vp, ci, vp]
        L.dgsp_spmm_csr_nnz.restype = ci
        L.dgsp_spmm_csr_nnz.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, ci, vp]
        L.dgsp_spmm_csr_auto.restype = ci
        L.dgsp_spmm_csr_auto.argtypes = [i64, i64, i64, ctypes.POINTER(Features), vp, vp, vp, vp, vp,
                                         ctypes.POINTER(ci), vp]
        L.dgsp_select_algo.restype = ci
        L.dgsp_select_algo.argtypes = [ctypes.POINTER(Features), i64]
        L.dgsp_get_thresholds.restype = None
        L.dgsp_get_thresholds.argtypes = [ctypes.POINTER(Thresholds)]
        L.dgsp_set_thresholds.restype = None
        L.dgsp_set_thresholds.argtypes = [ctypes.POINTER(Thresholds)]
        L.dgsp_features_from_rowptr_host.restype = ci
        L.dgsp_features_from_rowptr_host.argtypes = [i64, i64, vp, ctypes.POINTER(Features)]
        L.dgsp_features_from_csr_host.restype = ci
        L.dgsp_features_from_csr_host.argtypes = [i64, i64, vp, vp, ctypes.POINTER(Features)]
        L.dgsp_spmm_csr_phase.restype = ci
        L.dgsp_spmm_csr_phase.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, ci, ci, ctypes.POINTER(Features), vp]
        L.dgsp_features_from_csr_device.restype = ci
        L.dgsp_features_from_csr_device.argtypes = [i64, i64, vp, vp, vp, ctypes.POINTER(Features), vp]
        L.dgsp_features_from_csr_device_noalloc.restype = ci
        L.dgsp_features_from_csr_device_noalloc.argtypes = [i64, i64, vp, vp, ctypes.POINTER(Features), vp]
        L.dgsp_autotune.restype = ci
        L.dgsp_autotune.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, ctypes.POINTER(Features), ci,
                                    ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ci), vp]
        L.dgsp_spmm_csr_ld.restype = ci
        L.dgsp_spmm_csr_ld.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, i64, vp, i64, ci, ctypes.POINTER(Features), vp]
        L.dgsp_spmm_csr_axpby.restype = ci
        L.dgsp_spmm_csr_axpby.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, i64, vp, i64, ctypes.c_float, ctypes.c_float,
                                          ci, ctypes.POINTER(Features), vp]
        L.dgsp_spmm_csr_ablation.restype = ci
        L.dgsp_spmm_csr_ablation.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, ci, ci, ctypes.POINTER(Features), vp]
        L.dgsp_gather_probe.restype = ci
        L.dgsp_gather_probe.argtypes = [vp, vp, vp, i64, vp]
        L.dgsp_gather_probe_out_len.restype = i64
        L.dgsp_gather_probe_out_len.argtypes = []
        L.dgsp_spmm_csr_i64.restype = ci
        L.dgsp_spmm_csr_i64.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, ci, vp, i64, vp]
        L.dgsp_spmm_csr_i64_workspace_bytes.restype = i64
        L.dgsp_spmm_csr_i64_workspace_bytes.argtypes = [i64, i64]
        L.dgsp_floor_probe.restype = ci
        L.dgsp_floor_probe.argtypes = [ci, i64, i64, i64, vp, vp, vp, vp, vp]
        L.dgsp_floor_probe_out_len.restype = i64
        L.dgsp_floor_probe_out_len.argtypes = [ci, i64]
        L.dgsp_copy_f32.restype = ci
        L.dgsp_copy_f32.argtypes = [vp, vp, i64, vp]
        L.dgsp_algo_name.restype = ctypes.c_char_p
        L.dgsp_algo_name.argtypes = [ci]
        L.dgsp_status_string.restype = ctypes.c_char_p
        L.dgsp_status_string.argtypes = [ci]
        _lib = L
    return _lib


def _check(rc: int, what: str):
    if rc != OK:
        raise DgspError(f"{what}: {dgsp_status_string(rc)} (status {rc})")


def _ptr(t):
    return None if t is None or t.numel() == 0 else t.data_ptr()


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_device_tensors(M, K, N, rowptr, colidx, vals, X, Y):
    import torch
    for name, t, dt in (("rowptr", rowptr, torch.int32), ("colidx", colidx, torch.int32),
                        ("vals", vals, torch.float32), ("X", X, torch.float32), ("Y", Y, torch.float32)):
        if not t.is_cuda or t.dtype != dt or not t.is_contiguous():
            raise DgspError(f"{name} must be a contiguous {dt} tensor on the GPU")
    if rowptr.numel() != M + 1 or colidx.numel() != vals.numel():
        raise DgspError("rowptr needs M+1 entries; colidx and vals must have equal length")
    if X.numel() != K * N or Y.numel() != M * N:
        raise DgspError("X must hold K*N and Y M*N elements")


def dgsp_spmm_csr(M, K, N, rowptr, colidx, vals, X, Y, algo, stream=None):
    """``Y = A X`` with the kernel ``algo``; the entry count is read on the device."""
    _check_device_tensors(M, K, N, rowptr, colidx, vals, X, Y)
    rc = lib().dgsp_spmm_csr(M, K, N, _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), _ptr(Y),
                             int(algo), _stream(stream))
    _check(rc, "dgsp_spmm_csr")


def dgsp_spmm_csr_nnz(M, K, N, nnz, rowptr, colidx, vals, X, Y, algo, stream=None):
    """``Y = A X`` with the entry count given by the caller."""
    _check_device_tensors(M, K, N, rowptr, colidx, vals, X, Y)
    if nnz >= 0 and colidx.numel() < nnz:
        raise DgspError("colidx/vals shorter than nnz")
    rc = lib().dgsp_spmm_csr_nnz(M, K, N, int(nnz), _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), _ptr(Y),
                                 int(algo), _stream(stream))
    _check(rc, "dgsp_spmm_csr_nnz")


def dgsp_spmm_csr_i64(M, K, N, nnz, rowptr, colidx, vals, X, Y, algo=AUTO, workspace=None, stream=None):
    """``Y = A X`` with int64 row pointers (more than 2^31 stored entries).  ``workspace``: a uint8 GPU tensor of
    ``dgsp_spmm_csr_i64_workspace_bytes(M, nnz)`` bytes (made here if not given).  Waits once for the stream."""
    import torch
    if not rowptr.is_cuda or rowptr.dtype != torch.int64 or not rowptr.is_contiguous() or rowptr.numel() != M + 1:
        raise DgspError("rowptr must be a contiguous int64 GPU tensor of M+1 entries")
    for name, t, dt in (("colidx", colidx, torch.int32), ("vals", vals, torch.float32), ("X", X, torch.float32),
                        ("Y", Y, torch.float32)):
        if not t.is_cuda or t.dtype != dt or not t.is_contiguous():
            raise DgspError(f"{name} must be a contiguous {dt} tensor on the GPU")
    if colidx.numel() < nnz or vals.numel() < nnz or X.numel() != K * N or Y.numel() != M * N:
        raise DgspError("colidx and vals need nnz entries, X K*N and Y M*N elements")
    need = int(lib().dgsp_spmm_csr_i64_workspace_bytes(M, int(nnz)))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=rowptr.device)
    rc = lib().dgsp_spmm_csr_i64(M, K, N, int(nnz), _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), _ptr(Y), int(algo),
                                 _ptr(workspace), int(workspace.numel()), _stream(stream))
    _check(rc, "dgsp_spmm_csr_i64")


def dgsp_spmm_csr_phase(M, K, N, nnz, rowptr, colidx, vals, X, Y, algo, phase, features=None, stream=None):
    """One step of the multiplication (measurement aid): PHASE_PREPARE, PHASE_MAIN or PHASE_ALL."""
    _check_device_tensors(M, K, N, rowptr, colidx, vals, X, Y)
    rc = lib().dgsp_spmm_csr_phase(M, K, N, int(nnz), _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), _ptr(Y),
                                   int(algo), int(phase), ctypes.byref(features) if features is not None else None,
                                   _stream(stream))
    _check(rc, "dgsp_spmm_csr_phase")


def dgsp_spmm_csr_ld(M, K, N, nnz, rowptr, colidx, vals, X, Y, algo=AUTO, features=None, stream=None):
    """``Y = A X`` on 2-D views whose rows are ``stride(0)`` floats apart (``stride(1)`` must be 1):
    column slices of wider row-major tensors are taken as they are, nothing is copied."""
    import torch
    for name, t in (("X", X), ("Y", Y)):
        if not t.is_cuda or t.dtype != torch.float32 or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise DgspError(f"{name} must be a 2-D float32 GPU view with unit column stride")
    if X.shape != (K, N) or Y.shape != (M, N):
        raise DgspError("X must be K x N and Y M x N")
    ldx = X.stride(0) if K > 1 else max(N, X.stride(0))
    ldy = Y.stride(0) if M > 1 else max(N, Y.stride(0))
    rc = lib().dgsp_spmm_csr_ld(M, K, N, int(nnz), _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), int(ldx),
                                _ptr(Y), int(ldy), int(algo),
                                ctypes.byref(features) if features is not None else None, _stream(stream))
    _check(rc, "dgsp_spmm_csr_ld")


def dgsp_spmm_csr_axpby(M, K, N, nnz, rowptr, colidx, vals, X, Y, alpha=1.0, beta=0.0, algo=AUTO, features=None,
                        stream=None):
    """``Y = alpha * A X + beta * Y`` on 2-D views (rows ``stride(0)`` floats apart, unit column stride)."""
    import torch
    for name, t in (("X", X), ("Y", Y)):
        if not t.is_cuda or t.dtype != torch.float32 or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
            raise DgspError(f"{name} must be a 2-D float32 GPU view with unit column stride")
    if X.shape != (K, N) or Y.shape != (M, N):
        raise DgspError("X must be K x N and Y M x N")
    ldx = X.stride(0) if K > 1 else max(N, X.stride(0))
    ldy = Y.stride(0) if M > 1 else max(N, Y.stride(0))
    rc = lib().dgsp_spmm_csr_axpby(M, K, N, int(nnz), _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), int(ldx),
                                   _ptr(Y), int(ldy), float(alpha), float(beta), int(algo),
                                   ctypes.byref(features) if features is not None else None, _stream(stream))
    _check(rc, "dgsp_spmm_csr_axpby")


def dgsp_spmm_csr_ablation(M, K, N, nnz, rowptr, colidx, vals, X, Y, algo, switches, features=None, stream=None):
    """The multiplication with optimisations switched off (measurement aid): ABL_SCALAR_DENSE_LOADS,
    ABL_NO_SPARSE_STAGING."""
    _check_device_tensors(M, K, N, rowptr, colidx, vals, X, Y)
    rc = lib().dgsp_spmm_csr_ablation(M, K, N, int(nnz), _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), _ptr(Y),
                                      int(algo), int(switches),
                                      ctypes.byref(features) if features is not None else None, _stream(stream))
    _check(rc, "dgsp_spmm_csr_ablation")


def dgsp_features_from_csr_device(M, K, rowptr, colidx=None, workspace=None, stream=None) -> Features:
    """Row statistics of a matrix in device memory (waits for the result)."""
    import torch
    if workspace is None:
        workspace = torch.empty(FEATURES_WORKSPACE_BYTES // 8, dtype=torch.int64, device=rowptr.device)
    f = Features()
    rc = lib().dgsp_features_from_csr_device(M, K, _ptr(rowptr), _ptr(colidx) if colidx is not None else None,
                                             _ptr(workspace), ctypes.byref(f), _stream(stream))
    _check(rc, "dgsp_features_from_csr_device")
    return f


def dgsp_features_from_csr_device_noalloc(M, K, rowptr, colidx=None, stream=None) -> Features:
    """The same statistics with the scratch words in the library's static device array: the call allocates
    nothing and takes no workspace (calls that overlap on one GPU race; waits for the result)."""
    f = Features()
    rc = lib().dgsp_features_from_csr_device_noalloc(M, K, _ptr(rowptr), _ptr(colidx) if colidx is not None else None,
                                                     ctypes.byref(f), _stream(stream))
    _check(rc, "dgsp_features_from_csr_device_noalloc")
    return f


def dgsp_autotune(M, K, N, nnz, rowptr, colidx, vals, X, Y, features=None, reps=5, stream=None):
    """Times the four kernels on these buffers; returns (fastest algo, [ms of each kernel])."""
    _check_device_tensors(M, K, N, rowptr, colidx, vals, X, Y)
    ms = (ctypes.c_float * 4)()
    best = ctypes.c_int(-1)
    rc = lib().dgsp_autotune(M, K, N, int(nnz), _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), _ptr(Y),
                             ctypes.byref(features) if features is not None else None, int(reps), ms,
                             ctypes.byref(best), _stream(stream))
    _check(rc, "dgsp_autotune")
    return best.value, list(ms)


def dgsp_gather_probe(out, x, idx, n=None, stream=None):
    """``out[t] = sum x[idx[i]]`` (measurement aid: the pure gather rate of an index pattern)."""
    n = idx.numel() if n is None else n
    if out.numel() < dgsp_gather_probe_out_len():
        raise DgspError("out is shorter than dgsp_gather_probe_out_len()")
    rc = lib().dgsp_gather_probe(_ptr(out), _ptr(x), _ptr(idx), int(n), _stream(stream))
    _check(rc, "dgsp_gather_probe")


def dgsp_floor_probe_out_len(mode, N) -> int:
    return int(lib().dgsp_floor_probe_out_len(int(mode), int(N)))


def dgsp_floor_probe(mode, K, N, colidx, vals, X, out, stream=None):
    """The memory side of the kernels with no row logic (measurement aid); ``out`` receives per-thread partial sums
    whose total is the sum of all elements of ``A X``."""
    if out.numel() < dgsp_floor_probe_out_len(mode, N):
        raise DgspError("out is shorter than dgsp_floor_probe_out_len(mode, N) (or the mode does not offer this N)")
    rc = lib().dgsp_floor_probe(int(mode), int(colidx.numel()), int(K), int(N), _ptr(colidx), _ptr(vals), _ptr(X),
                                _ptr(out), _stream(stream))
    _check(rc, "dgsp_floor_probe")


def dgsp_gather_probe_out_len() -> int:
    return int(lib().dgsp_gather_probe_out_len())


def dgsp_spmm_csr_auto(M, K, N, features: Features, rowptr, colidx, vals, X, Y, stream=None) -> int:
    """Select by the rules, run, return the chosen algo."""
    _check_device_tensors(M, K, N, rowptr, colidx, vals, X, Y)
    chosen = ctypes.c_int(-1)
    rc = lib().dgsp_spmm_csr_auto(M, K, N, ctypes.byref(features), _ptr(rowptr), _ptr(colidx), _ptr(vals),
                                  _ptr(X), _ptr(Y), ctypes.byref(chosen), _stream(stream))
    _check(rc, "dgsp_spmm_csr_auto")
    return chosen.value


def dgsp_select_algo(features: Features, N: int) -> int:
    return int(lib().dgsp_select_algo(ctypes.byref(features), int(N)))


def dgsp_get_thresholds() -> Thresholds:
    t = Thresholds()
    lib().dgsp_get_thresholds(ctypes.byref(t))
    return t


def dgsp_set_thresholds(t: Thresholds) -> None:
    lib().dgsp_set_thresholds(ctypes.byref(t))


def dgsp_features_from_rowptr_host(M, K, rowptr_host) -> Features:
    """``rowptr_host``: a contiguous int32 numpy array (or CPU tensor) of M+1 entries."""
    import numpy as np
    a = np.ascontiguousarray(rowptr_host, dtype=np.int32)
    if a.size != M + 1:
        raise DgspError("rowptr needs M+1 entries")
    f = Features()
    rc = lib().dgsp_features_from_rowptr_host(M, K, a.ctypes.data, ctypes.byref(f))
    _check(rc, "dgsp_features_from_rowptr_host")
    return f


def dgsp_features_from_csr_host(M, K, rowptr_host, colidx_host) -> Features:
    """Row statistics plus ``col_span`` from host copies of rowptr and colidx."""
    import numpy as np
    rp = np.ascontiguousarray(rowptr_host, dtype=np.int32)
    ci = np.ascontiguousarray(colidx_host, dtype=np.int32)
    if rp.size != M + 1 or ci.size < int(rp[-1] if rp.size else 0):
        raise DgspError("rowptr needs M+1 entries and colidx rowptr[M]")
    f = Features()
    rc = lib().dgsp_features_from_csr_host(M, K, rp.ctypes.data, ci.ctypes.data if ci.size else None, ctypes.byref(f))
    _check(rc, "dgsp_features_from_csr_host")
    return f


def dgsp_copy_f32(dst, src, n=None, stream=None):
    n = dst.numel() if n is None else n
    rc = lib().dgsp_copy_f32(_ptr(dst), _ptr(src), int(n), _stream(stream))
    _check(rc, "dgsp_copy_f32")


def dgsp_algo_name(algo: int) -> str:
    return lib().dgsp_algo_name(int(algo)).decode()


def dgsp_status_string(status: int) -> str:
    return lib().dgsp_status_string(int(status)).decode()


class DeviceCsr:
    """A CSR matrix resident in GPU memory (plumbing for tests and benchmarks)."""

    def __init__(self, A, device="cuda:0"):
        import torch
        self.M, self.K, self.nnz = A.M, A.K, A.nnz
        self.rowptr = torch.from_numpy(A.rowptr).to(device)
        self.colidx = torch.from_numpy(A.colidx).to(device)
        self.vals = torch.from_numpy(A.vals).to(device)
        self.features = dgsp_features_from_csr_host(A.M, A.K, A.rowptr, A.colidx)
        self.tuned = {}        # N -> kernel found fastest by autotune()

    @classmethod
    def from_device(cls, M, K, rowptr, colidx, vals):
        """Wraps CSR arrays that already live on the GPU (int32 ``rowptr`` / ``colidx``, float32 ``vals``; other
        integer or float types are converted once).  The row statistics are computed on the device."""
        import torch
        self = cls.__new__(cls)
        self.M, self.K = int(M), int(K)
        self.rowptr = rowptr.to(torch.int32).contiguous()
        self.colidx = colidx.to(torch.int32).contiguous()
        self.vals = vals.to(torch.float32).contiguous()
        self.nnz = int(self.colidx.numel())
        self.features = dgsp_features_from_csr_device(self.M, self.K, self.rowptr, self.colidx if self.nnz else None)
        self.tuned = {}
        return self

    @classmethod
    def from_torch_sparse_csr(cls, t):
        """From a ``torch.sparse_csr_tensor`` on the GPU."""
        return cls.from_device(t.shape[0], t.shape[1], t.crow_indices(), t.col_indices(), t.values())

    def autotune(self, X, reps=5, Y=None):
        """Times the four kernels for this matrix and this width of X and remembers the winner:
        later ``spmm(X, algo=AUTO)`` calls with the same width use it instead of the rules."""
        import torch
        N = X.shape[1] if X.dim() == 2 else 1
        if Y is None:
            Y = torch.empty((self.M, N), dtype=torch.float32, device=X.device)
        best, ms = dgsp_autotune(self.M, self.K, N, self.nnz, self.rowptr, self.colidx, self.vals, X, Y,
                                 self.features, reps)
        self.tuned[N] = best
        return best, ms

    def spmm(self, X, algo=AUTO, Y=None, use_nnz=True, stream=None):
        """Y = A X.  ``algo=AUTO`` applies the selection rules to this matrix's features."""
        import torch
        N = X.shape[1] if X.dim() == 2 else 1
        if Y is None:
            Y = torch.empty((self.M, N), dtype=torch.float32, device=X.device)
        if algo == AUTO and N in getattr(self, "tuned", {}):
            algo = self.tuned[N]
        if algo == AUTO:
            dgsp_spmm_csr_auto(self.M, self.K, N, self.features, self.rowptr, self.colidx, self.vals, X, Y, stream)
        elif use_nnz:
            # a named kernel with this matrix's hints (entry count, column span)
            dgsp_spmm_csr_phase(self.M, self.K, N, self.nnz, self.rowptr, self.colidx, self.vals, X, Y, algo,
                                PHASE_ALL, self.features, stream)
        else:
            dgsp_spmm_csr(self.M, self.K, N, self.rowptr, self.colidx, self.vals, X, Y, algo, stream)
        return Y
