"""Seeded synthetic inputs for the matrix chain D = A(BC).

This module only *generates data*: sparsity patterns, values and dense operands with the
shapes and structure of the five benchmark configurations.  It holds none of the method's
arithmetic (no products, no scheduling) and is the one module that both the CPU oracle's
tests and the GPU path's tests / bench use, so that both sides see identical inputs.

The paper evaluates on SuiteSparse matrices of two families (SPD / PDE-like and graph
matrices, Section 4.1 "Matrix Dataset") with 32, 64 or 128 dense columns in single and double
precision (Section 4.1 "Environment").  The matrices here are synthetic stand-ins for those
families: banded and 2D/3D Laplacian matrices for the SPD family, R-MAT graphs for the graph
family.

Every generator returns plain numpy arrays.  CSR matrices are `Csr` named tuples with int32
`rowptr`/`colidx` and values in the configuration's precision.
"""
from __future__ import annotations

from typing import NamedTuple, Optional

import numpy as np


class Csr(NamedTuple):
    n_rows: int
    n_cols: int
    rowptr: np.ndarray   # int32 [n_rows + 1]
    colidx: np.ndarray   # int32 [nnz]
    vals: np.ndarray     # float32 / float64 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


class Problem(NamedTuple):
    name: str
    kind: str                 # "gemm_spmm" (dense B) or "spmm_spmm" (CSR B)
    dtype: np.dtype
    A: Csr
    B: object                 # np.ndarray [n, bCol] or Csr
    C: np.ndarray             # [bCol, cCol]
    b_is_A: bool = False      # SpMM-SpMM with B the same matrix as A

    @property
    def n(self) -> int:
        return self.A.n_rows

    @property
    def bcol(self) -> int:
        return self.C.shape[0]

    @property
    def ccol(self) -> int:
        return self.C.shape[1]


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def _csr_from_coo(n_rows: int, n_cols: int, rows: np.ndarray, cols: np.ndarray,
                  vals: np.ndarray, dtype) -> Csr:
    """Rows/cols must already be free of duplicates; entries are sorted by (row, col)."""
    order = np.lexsort((cols, rows))
    rows = rows[order]
    cols = cols[order]
    vals = vals[order]
    counts = np.bincount(rows, minlength=n_rows)
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    assert rowptr[-1] < 2 ** 31
    return Csr(n_rows, n_cols, rowptr.astype(np.int32), cols.astype(np.int32),
               np.ascontiguousarray(vals.astype(dtype)))


# --------------------------------------------------------------------------- patterns

def banded(n: int, half_bandwidth: int, dtype, seed: int, ones: bool = False) -> Csr:
    """Full band |i-j| <= h clipped at the matrix edges; values U(-1,1) (or all ones)."""
    h = half_bandwidth
    offs = np.arange(-h, h + 1, dtype=np.int64)
    rows = np.repeat(np.arange(n, dtype=np.int64), offs.size)
    cols = rows + np.tile(offs, n)
    keep = (cols >= 0) & (cols < n)
    rows, cols = rows[keep], cols[keep]
    if ones:
        vals = np.ones(rows.size)
    else:
        vals = _rng(seed).uniform(-1.0, 1.0, size=rows.size)
    return _csr_from_coo(n, n, rows, cols, vals, dtype)


def laplacian_2d(g: int, dtype) -> Csr:
    """5-point Laplacian on a g x g grid, natural ordering (x fastest), Dirichlet truncation:
    diagonal 4, existing neighbours -1."""
    n = g * g
    idx = np.arange(n, dtype=np.int64)
    x = idx % g
    y = idx // g
    r = [idx]
    c = [idx]
    v = [np.full(n, 4.0)]
    for mask, off in ((x > 0, -1), (x < g - 1, 1), (y > 0, -g), (y < g - 1, g)):
        r.append(idx[mask])
        c.append(idx[mask] + off)
        v.append(np.full(int(mask.sum()), -1.0))
    return _csr_from_coo(n, n, np.concatenate(r), np.concatenate(c), np.concatenate(v), dtype)


def laplacian_3d(g: int, dtype) -> Csr:
    """7-point Laplacian on a g^3 grid, natural ordering (x fastest, then y, then z):
    diagonal 6, existing neighbours -1."""
    n = g * g * g
    idx = np.arange(n, dtype=np.int64)
    x = idx % g
    y = (idx // g) % g
    z = idx // (g * g)
    r = [idx]
    c = [idx]
    v = [np.full(n, 6.0)]
    for mask, off in ((x > 0, -1), (x < g - 1, 1), (y > 0, -g), (y < g - 1, g),
                      (z > 0, -g * g), (z < g - 1, g * g)):
        r.append(idx[mask])
        c.append(idx[mask] + off)
        v.append(np.full(int(mask.sum()), -1.0))
    return _csr_from_coo(n, n, np.concatenate(r), np.concatenate(c), np.concatenate(v), dtype)


def rmat_edges(scale: int, n_draws: int, seed: int,
               a: float = 0.57, b: float = 0.19, c: float = 0.19) -> tuple:
    """Draw `n_draws` directed R-MAT edges on 2^scale vertices: one quadrant choice
    (a, b, c, d = 1-a-b-c) per bit, most significant bit first.  No vertex relabelling."""
    rng = _rng(seed)
    src = np.zeros(n_draws, dtype=np.int64)
    dst = np.zeros(n_draws, dtype=np.int64)
    for _ in range(scale):
        u = rng.random(n_draws)
        right = ((u >= a) & (u < a + b)) | (u >= a + b + c)      # quadrants b and d
        down = u >= a + b                                       # quadrants c and d
        src = (src << 1) | down
        dst = (dst << 1) | right
    return src, dst


def rmat_symmetric_pattern(scale: int, n_draws: int, seed: int) -> tuple:
    """Undirected simple graph from R-MAT draws: self-loops dropped, edges symmetrised and
    deduplicated.  Returns (lo, hi) arrays of the unique undirected edges with lo < hi."""
    src, dst = rmat_edges(scale, n_draws, seed)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    lo = np.minimum(src, dst)
    hi = np.maximum(src, dst)
    n = 1 << scale
    key = np.unique(lo * n + hi)
    return key // n, key % n


def rmat_symmetric(scale: int, n_draws: int, dtype, seed: int) -> Csr:
    """Symmetric R-MAT matrix with one U(0,1) value per undirected edge."""
    lo, hi = rmat_symmetric_pattern(scale, n_draws, seed)
    n = 1 << scale
    w = _rng(seed + 7919).uniform(0.0, 1.0, size=lo.size)
    rows = np.concatenate([lo, hi])
    cols = np.concatenate([hi, lo])
    vals = np.concatenate([w, w])
    return _csr_from_coo(n, n, rows, cols, vals, dtype)


def gcn_normalised(scale: int, n_draws: int, dtype, seed: int) -> Csr:
    """GCN propagation matrix deg^-1/2 (Adj + I) deg^-1/2 of the symmetric R-MAT graph, where
    deg holds the row sums of Adj + I (0/1 adjacency)."""
    lo, hi = rmat_symmetric_pattern(scale, n_draws, seed)
    n = 1 << scale
    diag = np.arange(n, dtype=np.int64)
    rows = np.concatenate([lo, hi, diag])
    cols = np.concatenate([hi, lo, diag])
    deg = np.bincount(rows, minlength=n).astype(np.float64)
    vals = 1.0 / np.sqrt(deg[rows] * deg[cols])
    return _csr_from_coo(n, n, rows, cols, vals, dtype)


def uniform_random_csr(n_rows: int, n_cols: int, nnz_per_row: int, dtype, seed: int) -> Csr:
    """Exactly `nnz_per_row` distinct uniform-random columns per row, sorted, values U(-1,1)."""
    rng = _rng(seed)
    k = nnz_per_row
    assert k <= n_cols
    cols = rng.integers(0, n_cols, size=(n_rows, k), dtype=np.int64)
    cols.sort(axis=1)
    # redraw rows that contain a repeated column until every row is duplicate-free
    while True:
        bad = np.nonzero((cols[:, 1:] == cols[:, :-1]).any(axis=1))[0]
        if bad.size == 0:
            break
        fresh = rng.integers(0, n_cols, size=(bad.size, k), dtype=np.int64)
        fresh.sort(axis=1)
        cols[bad] = fresh
    vals = rng.uniform(-1.0, 1.0, size=(n_rows, k))
    rowptr = (np.arange(n_rows + 1, dtype=np.int64) * k).astype(np.int32)
    return Csr(n_rows, n_cols, rowptr, cols.reshape(-1).astype(np.int32),
               np.ascontiguousarray(vals.reshape(-1).astype(dtype)))


def random_pattern_csr(n_rows: int, n_cols: int, density: float, dtype, seed: int,
                       sort_cols: bool = True, duplicates: bool = False,
                       empty_row_prob: float = 0.0, int_values: bool = False) -> Csr:
    """Small random CSR for tests: optional unsorted columns, duplicate entries, empty rows and
    small-integer values (every summation order is then exact)."""
    rng = _rng(seed)
    rowptr = [0]
    cols = []
    for _ in range(n_rows):
        if rng.random() < empty_row_prob:
            rowptr.append(rowptr[-1])
            continue
        m = rng.binomial(n_cols, density)
        c = rng.choice(n_cols, size=m, replace=False)
        if duplicates and m > 0:
            extra = rng.choice(c, size=max(1, m // 3))
            c = np.concatenate([c, extra])
        if sort_cols:
            c = np.sort(c)
        else:
            c = rng.permutation(c)
        cols.append(c)
        rowptr.append(rowptr[-1] + c.size)
    colidx = np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32)
    if int_values:
        vals = rng.integers(-2, 3, size=colidx.size).astype(dtype)
    else:
        vals = rng.uniform(-1.0, 1.0, size=colidx.size).astype(dtype)
    return Csr(n_rows, n_cols, np.asarray(rowptr, dtype=np.int32), colidx, vals)


def random_local_csr(n: int, width: int, nnz_per_row: int, far_prob: float, dtype, seed: int,
                     int_values: bool = False, empty_row_prob: float = 0.1) -> Csr:
    """Small square test matrix whose rows mostly stay within `width` of the diagonal, so that
    consecutive tiles fuse many rows, while a fraction `far_prob` of the rows also holds one
    far-away column.  Columns are unsorted and may repeat."""
    rng = _rng(seed)
    rowptr = [0]
    cols = []
    for j in range(n):
        if rng.random() < empty_row_prob:
            rowptr.append(rowptr[-1])
            continue
        lo, hi = max(0, j - width), min(n, j + width + 1)
        c = rng.integers(lo, hi, size=nnz_per_row)
        if rng.random() < far_prob:
            c = np.append(c, rng.integers(0, n))
        cols.append(c)
        rowptr.append(rowptr[-1] + c.size)
    colidx = np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32)
    if int_values:
        vals = rng.integers(-2, 3, size=colidx.size).astype(dtype)
    else:
        vals = rng.uniform(-1.0, 1.0, size=colidx.size).astype(dtype)
    return Csr(n, n, np.asarray(rowptr, dtype=np.int32), colidx, vals)


def random_hub_csr(n: int, dtype, seed: int, n_hubs: int = 3, hub_len: int = 300,
                   int_values: bool = True) -> Csr:
    """Small square test matrix with the shape of a graph matrix: most rows hold a few columns
    anywhere in the matrix (unsorted, may repeat), `n_hubs` rows hold `hub_len` columns, about a
    fifth of the rows hold only their diagonal entry and about a tenth are empty."""
    rng = _rng(seed)
    hubs = set(rng.choice(n, size=min(n_hubs, n), replace=False).tolist())
    rowptr = [0]
    cols = []
    for j in range(n):
        u = rng.random()
        if j in hubs:
            c = rng.integers(0, n, size=hub_len)
        elif u < 0.1:
            c = np.zeros(0, dtype=np.int64)
        elif u < 0.3:
            c = np.array([j])
        else:
            c = rng.integers(0, n, size=int(rng.integers(1, 12)))
        cols.append(c)
        rowptr.append(rowptr[-1] + c.size)
    colidx = np.concatenate(cols).astype(np.int32)
    if int_values:
        vals = rng.integers(-2, 3, size=colidx.size).astype(dtype)
    else:
        vals = rng.uniform(-1.0, 1.0, size=colidx.size).astype(dtype)
    return Csr(n, n, np.asarray(rowptr, dtype=np.int32), colidx, vals)


def dense_normal(rows: int, cols: int, dtype, seed: int, std: float = 1.0) -> np.ndarray:
    return np.ascontiguousarray((_rng(seed).standard_normal((rows, cols)) * std).astype(dtype))


def dense_uniform(rows: int, cols: int, dtype, seed: int, bound: float) -> np.ndarray:
    return np.ascontiguousarray(_rng(seed).uniform(-bound, bound, size=(rows, cols)).astype(dtype))


def dense_small_int(rows: int, cols: int, dtype, seed: int) -> np.ndarray:
    return np.ascontiguousarray(_rng(seed).integers(-2, 3, size=(rows, cols)).astype(dtype))


# --------------------------------------------------------------------------- the five configs

N_CONFIGS = 5


def config(cfg: int, scale_down: Optional[int] = None, width: Optional[int] = None,
           dtype=None) -> Problem:
    """The benchmark configurations, numbered 1..5.  Seeds are 1000 + cfg.

    `scale_down` (tests only) shrinks the problem while keeping its structure: it is the grid
    edge for configs 2 and 4, the R-MAT scale for configs 3 and 5, and n for config 1.
    `width` and `dtype` move a configuration over the paper's experiment grid (Section 4.1:
    bCol = cCol in {32, 64, 128}, single and double precision): width replaces bCol and cCol of a
    dense B and cCol of a sparse one, dtype the precision; matrices and seeds stay the same.
    """
    seed = 1000 + cfg
    tag = lambda dt: "fp32" if np.dtype(dt) == np.float32 else "fp64"
    if cfg == 1:
        n = scale_down or 4096
        dt = dtype or np.float64
        w = width or 32
        A = banded(n, 8, dt, seed)
        B = dense_normal(n, w, dt, seed + 1)
        C = dense_normal(w, w, dt, seed + 2)
        return Problem(f"cfg1 GeMM-SpMM {tag(dt)} band h=8", "gemm_spmm", np.dtype(dt), A, B, C)
    if cfg == 2:
        g = scale_down or 512
        dt = dtype or np.float32
        w = width or 64
        A = laplacian_2d(g, dt)
        B = dense_normal(g * g, w, dt, seed + 1)
        C = dense_normal(w, w, dt, seed + 2, std=float(1.0 / np.sqrt(w)))      # variance 1/w
        return Problem(f"cfg2 GeMM-SpMM {tag(dt)} 2D Laplacian", "gemm_spmm", np.dtype(dt), A, B, C)
    if cfg == 3:
        s = scale_down or 20
        dt = dtype or np.float32
        w = width or 128
        n = 1 << s
        A = gcn_normalised(s, 8 * n, dt, seed)
        B = dense_normal(n, w, dt, seed + 1)
        C = dense_uniform(w, w, dt, seed + 2, bound=float(np.sqrt(6.0 / (2 * w))))
        return Problem(f"cfg3 GeMM-SpMM {tag(dt)} GCN R-MAT", "gemm_spmm", np.dtype(dt), A, B, C)
    if cfg == 4:
        g = scale_down or 64
        dt = dtype or np.float64
        A = laplacian_3d(g, dt)
        C = dense_normal(g ** 3, width or 64, dt, seed + 2)
        return Problem(f"cfg4 SpMM-SpMM {tag(dt)} 3D Laplacian", "spmm_spmm", np.dtype(dt), A, A, C,
                       b_is_A=True)
    if cfg == 5:
        s = scale_down or 20
        dt = dtype or np.float32
        n = 1 << s
        A = rmat_symmetric(s, 8 * n, dt, seed)
        B = uniform_random_csr(n, n, 8, dt, seed + 1)
        C = dense_normal(n, width or 32, dt, seed + 2)
        return Problem(f"cfg5 SpMM-SpMM {tag(dt)} R-MAT x random", "spmm_spmm", np.dtype(dt), A, B, C)
    raise ValueError(f"config must be 1..{N_CONFIGS}")


def useful_flops(p: Problem) -> int:
    """FLOP count of the unfused code, used for every implementation (Section 4.1)."""
    if p.kind == "gemm_spmm":
        first = 2 * p.n * p.bcol * p.ccol
    else:
        first = 2 * p.B.nnz * p.ccol
    return first + 2 * p.A.nnz * p.ccol
