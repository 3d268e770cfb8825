"""Seeded synthetic CSR matrices and dense operands (host side, numpy only).

These generators stand in for the matrix collections the paper measured on
(Section 3.1: a public sparse-matrix collection; Section 2.1.2: a 27-matrix
R-MAT micro-benchmark whose parameters are not printed).  They hold none of the
method's arithmetic: no products, no row sums of products, no reductions over
``A`` and ``X`` together.  Both the CPU oracle's tests and the GPU tests call
them, so that the two sides see identical inputs.

Every generator is a pure function of its arguments and ``seed``: draws are
taken from ``numpy.random.default_rng(seed)`` in a fixed, documented order.
All matrices are CSR with int32 ``rowptr`` (M+1) and ``colidx`` (nnz), fp32
``vals`` (nnz), zero-based, column indices ascending and unique inside a row.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class CsrMatrix:
    M: int
    K: int
    rowptr: np.ndarray   # int32, M+1
    colidx: np.ndarray   # int32, nnz
    vals: np.ndarray     # float32, nnz
    name: str = ""
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def row_lengths(self) -> np.ndarray:
        return np.diff(self.rowptr.astype(np.int64))

    def k_touched(self) -> int:
        """Number of distinct columns that hold at least one stored entry."""
        if "k_touched" not in self.meta:
            seen = np.zeros(self.K, dtype=bool)
            seen[self.colidx] = True
            self.meta["k_touched"] = int(seen.sum())
        return self.meta["k_touched"]

    def stats(self) -> dict:
        lens = self.row_lengths()
        mean = float(lens.mean()) if lens.size else 0.0
        std = float(lens.std()) if lens.size else 0.0
        return dict(M=self.M, K=self.K, nnz=self.nnz, mean=mean, std=std,
                    cv=(std / mean if mean > 0 else 0.0),
                    max=int(lens.max()) if lens.size else 0,
                    empty_frac=float((lens == 0).mean()) if lens.size else 0.0)


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------

def _rowptr_from_lens(lens: np.ndarray) -> np.ndarray:
    rowptr = np.zeros(lens.size + 1, dtype=np.int64)
    np.cumsum(lens, out=rowptr[1:])
    if rowptr[-1] >= 2 ** 31:
        raise ValueError("nnz does not fit int32 indexing")
    return rowptr.astype(np.int32)


def _distinct_columns(lens: np.ndarray, K: int, rng: np.random.Generator) -> np.ndarray:
    """For every row i, ``lens[i]`` distinct columns uniform on [0, K), ascending.

    Draw with replacement, then redraw only the colliding entries until none
    collide; rows asking for more than K/4 columns take a per-row permutation
    instead (only tiny test matrices reach that branch).
    """
    lens = np.asarray(lens, dtype=np.int64)
    M = lens.size
    nnz = int(lens.sum())
    rows = np.repeat(np.arange(M, dtype=np.int64), lens)
    cols = rng.integers(0, K, size=nnz, dtype=np.int64) if nnz else np.zeros(0, np.int64)
    dense_rows = np.flatnonzero(lens > K // 4)
    if dense_rows.size:
        starts = np.concatenate(([0], np.cumsum(lens)))[:-1]
        for i in dense_rows:
            cols[starts[i]:starts[i] + lens[i]] = rng.permutation(K)[: lens[i]]
    for _ in range(200):
        key = rows * K + cols
        order = np.argsort(key, kind="stable")
        sk = key[order]
        dup = np.zeros(nnz, dtype=bool)
        dup[order[1:]] = sk[1:] == sk[:-1]
        ndup = int(dup.sum())
        if ndup == 0:
            break
        cols[dup] = rng.integers(0, K, size=ndup, dtype=np.int64)
    else:  # pragma: no cover
        raise RuntimeError("column de-duplication did not converge")
    key = rows * K + cols
    key.sort()
    return (key % K).astype(np.int32)


def _from_lens(lens, K, rng, name, value_fn, meta=None) -> CsrMatrix:
    lens = np.clip(np.asarray(lens, dtype=np.int64), 0, K)
    rowptr = _rowptr_from_lens(lens)
    colidx = _distinct_columns(lens, K, rng)
    vals = value_fn(int(rowptr[-1]))
    return CsrMatrix(int(lens.size), int(K), rowptr, colidx, vals.astype(np.float32), name, meta or {})


# --------------------------------------------------------------------------
# the benchmark configurations
# --------------------------------------------------------------------------

def poisson_csr(M=4096, K=4096, mean=8.0, seed=0) -> CsrMatrix:
    """Tiny-SpMM config: row lengths Poisson(mean) clipped to [0, K]; columns
    distinct uniform; values U(-1, 1).  Draw order: lengths, columns, values."""
    rng = np.random.default_rng(seed)
    lens = rng.poisson(mean, size=M)
    return _from_lens(lens, K, rng, f"poisson{mean:g}_M{M}_s{seed}",
                      lambda n: rng.uniform(-1.0, 1.0, size=n),
                      dict(kind="poisson", mean=mean, seed=seed))


def rmat_csr(scale=20, avg_degree=16, abcd=(0.57, 0.19, 0.19, 0.05), seed=0,
             values="uniform01") -> CsrMatrix:
    """R-MAT graph on 2**scale vertices with avg_degree * 2**scale edge draws.

    Each edge picks one quadrant per level (``scale`` independent choices, no
    noise, no vertex permutation); row = source, column = destination.
    Duplicate edges are merged (one entry kept), self-loops kept, columns
    ascending.  ``values``: ``"uniform01"`` draws U(0,1) after merging (the
    power-law SpMV config), ``"rownorm"`` sets every entry of row i to
    1/len_i (the GNN-style config), ``"ones"`` sets 1.0.
    Draw order: one U(0,1) vector per level (most significant bit first), then
    the values.
    """
    a, b, c, d = abcd
    rng = np.random.default_rng(seed)
    n = 1 << scale
    E = int(avg_degree) * n
    row = np.zeros(E, dtype=np.int64)
    col = np.zeros(E, dtype=np.int64)
    for _ in range(scale):
        u = rng.random(E, dtype=np.float32)
        rbit = u >= np.float32(a + b)
        cbit = ((u >= np.float32(a)) & (u < np.float32(a + b))) | (u >= np.float32(a + b + c))
        row = (row << 1) | rbit
        col = (col << 1) | cbit
    key = np.unique(row * n + col)
    row = key // n
    colidx = (key % n).astype(np.int32)
    lens = np.bincount(row, minlength=n)
    rowptr = _rowptr_from_lens(lens)
    nnz = int(rowptr[-1])
    if values == "uniform01":
        vals = rng.random(nnz, dtype=np.float32)
    elif values == "rownorm":
        vals = (1.0 / np.repeat(lens, lens).astype(np.float64)).astype(np.float32)
    elif values == "ones":
        vals = np.ones(nnz, dtype=np.float32)
    else:
        raise ValueError(values)
    return CsrMatrix(n, n, rowptr, colidx, vals, f"rmat{scale}_d{avg_degree}_{values}_s{seed}",
                     dict(kind="rmat", scale=scale, avg_degree=avg_degree, abcd=abcd,
                          seed=seed, values=values, edge_draws=E))


def stencil27_csr(n=128, seed=0, values="normal_diag27") -> CsrMatrix:
    """3-D 27-point stencil on an n^3 grid, no periodic wrap.

    Row id = (z*n + y)*n + x; neighbours (dz,dy,dx) in {-1,0,1}^3 that fall
    inside the grid, which (taken in that lexicographic order) are already in
    ascending column order.  ``values``: ``"normal_diag27"`` draws N(0,1) per
    entry and adds 27 to the diagonal entry; ``"ones"`` sets 1.0.
    nnz = (3n-2)^3; row lengths lie in {8, 12, 18, 27}.
    """
    rng = np.random.default_rng(seed)
    idx = np.arange(n, dtype=np.int32)
    z, y, x = np.meshgrid(idx, idx, idx, indexing="ij")
    z, y, x = z.ravel(), y.ravel(), x.ravel()
    M = n ** 3
    cols = np.empty((M, 27), dtype=np.int32)
    valid = np.empty((M, 27), dtype=bool)
    diag = np.zeros((M, 27), dtype=bool)
    j = 0
    for dz in (-1, 0, 1):
        for dy in (-1, 0, 1):
            for dx in (-1, 0, 1):
                zz, yy, xx = z + dz, y + dy, x + dx
                ok = (zz >= 0) & (zz < n) & (yy >= 0) & (yy < n) & (xx >= 0) & (xx < n)
                valid[:, j] = ok
                cols[:, j] = (zz * n + yy) * n + xx
                if dz == 0 and dy == 0 and dx == 0:
                    diag[:, j] = True
                j += 1
    lens = valid.sum(axis=1)
    rowptr = _rowptr_from_lens(lens)
    colidx = cols[valid]
    is_diag = diag[valid]
    nnz = int(rowptr[-1])
    if values == "normal_diag27":
        vals = rng.standard_normal(nnz, dtype=np.float32)
        vals[is_diag] += np.float32(27.0)
    elif values == "ones":
        vals = np.ones(nnz, dtype=np.float32)
    else:
        raise ValueError(values)
    return CsrMatrix(M, M, rowptr, colidx.astype(np.int32), vals, f"stencil27_n{n}_{values}_s{seed}",
                     dict(kind="stencil27", n=n, seed=seed, values=values))


def zipf_truncation(mean: float, alpha: float = 1.5, kmax: int = 1 << 18) -> int:
    """Smallest C such that the law P(len=k) ~ k^-alpha on {1..C} has mean >= ``mean``."""
    k = np.arange(1, kmax + 1, dtype=np.float64)
    w = k ** (-alpha)
    means = np.cumsum(k * w) / np.cumsum(w)
    C = int(np.searchsorted(means, mean, side="left")) + 1
    return min(C, kmax)


SWEEP_DISTS = ("fixed", "poisson", "lognormal", "zipf")
SWEEP_MEANS = (4, 16, 64)
SWEEP_SEEDS = (0, 1)
SWEEP_NS = (1, 2, 4, 8, 16, 32, 64, 128, 256, 512)


def sweep_csr(M=1 << 18, mean=16, dist="poisson", seed=0) -> CsrMatrix:
    """One matrix of the selector sweep (square, K = M).

    Row-length laws, each with expectation ``mean``:
      fixed      every row has exactly ``mean`` entries;
      poisson    Poisson(mean);
      lognormal  round(exp(ln(mean) - 1/2 + Z)), Z ~ N(0,1)  (sigma = 1);
      zipf       P(len = k) ~ k^-1.5 on {1..C}, C chosen so the law's mean is
                 ``mean`` (a Zipf(1.5) law capped only at K has mean ~ 392, so
                 the cap is where the mean is set).
    Lengths are clipped to [0, K]; columns distinct uniform; values U(-1,1).
    Draw order: lengths, columns, values.
    """
    rng = np.random.default_rng([seed, SWEEP_DISTS.index(dist), int(mean)])
    K = M
    if dist == "fixed":
        lens = np.full(M, int(mean), dtype=np.int64)
    elif dist == "poisson":
        lens = rng.poisson(mean, size=M)
    elif dist == "lognormal":
        lens = np.rint(np.exp(np.log(mean) - 0.5 + rng.standard_normal(M))).astype(np.int64)
    elif dist == "zipf":
        C = zipf_truncation(mean, 1.5, K)
        k = np.arange(1, C + 1, dtype=np.float64)
        cdf = np.cumsum(k ** -1.5)
        cdf /= cdf[-1]
        lens = np.searchsorted(cdf, rng.random(M), side="left") + 1
        lens = np.minimum(lens, C)
    else:
        raise ValueError(dist)
    return _from_lens(lens, K, rng, f"sweep_{dist}_mu{mean}_M{M}_s{seed}",
                      lambda n: rng.uniform(-1.0, 1.0, size=n),
                      dict(kind="sweep", dist=dist, mean=mean, seed=seed))


def sweep_matrices(M=1 << 18):
    """Yield the 24 sweep matrices (3 means x 4 laws x 2 seeds), lazily."""
    for mean in SWEEP_MEANS:
        for dist in SWEEP_DISTS:
            for seed in SWEEP_SEEDS:
                yield sweep_csr(M, mean, dist, seed)


HOLDOUT_LAWS = ("poisson9", "pareto", "alike27", "bursts", "one_giant", "tile_widths", "half_empty")


def holdout_law_csr(law: str, M=1 << 18, seed=0) -> CsrMatrix:
    """Matrices for scoring the selection rules on row-length laws they were NOT fitted on (the sweep's four laws
    are what the thresholds come from): Poisson(9); a heavy Pareto tail; all rows 27 long; long empty stretches with
    short bursts; Poisson(3) with one 20 000-entry row; lengths around the wave and tile widths (0 ... 257); Poisson(5)
    with the second half of the rows empty.  K = M, distinct uniform columns, values U(-1,1).
    Draw order: lengths, columns, values."""
    rng = np.random.default_rng([seed, 0x401d, HOLDOUT_LAWS.index(law)])
    if law == "poisson9":
        lens = rng.poisson(9.0, size=M)
    elif law == "pareto":
        lens = np.floor(rng.pareto(1.2, size=M) * 6.0).astype(np.int64)
    elif law == "alike27":
        lens = np.full(M, 27)
    elif law == "bursts":
        lens = np.zeros(M, dtype=np.int64)
        hot = rng.random(M) < 0.02
        lens[hot] = rng.integers(1, 20, size=int(hot.sum()))
    elif law == "one_giant":
        lens = rng.poisson(3.0, size=M)
        lens[int(rng.integers(0, M))] = 20000
    elif law == "tile_widths":
        lens = rng.choice([0, 1, 63, 64, 65, 127, 128, 129, 255, 256, 257], size=M)
    elif law == "half_empty":
        lens = rng.poisson(5.0, size=M)
        lens[M // 2:] = 0
    else:
        raise ValueError(law)
    return _from_lens(np.minimum(lens, M), M, rng, f"holdout_{law}_M{M}_s{seed}",
                      lambda n: rng.uniform(-1.0, 1.0, size=n), dict(kind="holdout", law=law, seed=seed))


def csr_from_lens(lens, K, seed=0, name="custom") -> CsrMatrix:
    """CSR with the given row lengths, distinct uniform columns, values U(-1,1)."""
    rng = np.random.default_rng(seed)
    return _from_lens(lens, K, rng, name, lambda n: rng.uniform(-1.0, 1.0, size=n),
                      dict(kind="custom", seed=seed))


def dense_matrix(K: int, N: int, dist="uniform", seed=0) -> np.ndarray:
    """Row-major K x N fp32 operand: ``"uniform"`` = U(-1,1), ``"normal"`` = N(0,1)."""
    rng = np.random.default_rng([seed, 0x5eed, N])
    if dist == "uniform":
        return rng.uniform(-1.0, 1.0, size=(K, N)).astype(np.float32)
    if dist == "normal":
        return rng.standard_normal((K, N), dtype=np.float32)
    raise ValueError(dist)
