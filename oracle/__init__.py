"""CPU oracle for tile fusion of D = A(BC)  --  TEST INFRASTRUCTURE, not part of the product.

Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may import
this package.  It shares no code with the GPU path (`paper_2407_00243_amd`) and never
imports it.

Numerics (`tf_oracle.c`, wrapped here): the unfused definition D1 = BC, D = A D1 of the paper's
Section 1 (Eq. 1) in scalar fp64 with a fixed summation order, plus the error normaliser
W = |A| (|B| |C|) obtained by running the very same loops on the absolute values.

Schedule (`schedule.py`): a set-based restatement of Algorithm 1 (coarse tile fusion and tile
splitting) and an implementation-free validator of any fused schedule.

Pins (tests/test_oracle_*.py): dense brute force in extended precision, A = I, associativity,
exact small-integer inputs, closed forms for banded / Laplacian / GCN matrices, scipy.sparse
on special cases, closed-form fused-row counts; the transposed-C first operation against a
hand-worked 1 x 2 example and against the pinned plain one on an explicitly transposed array.  The data-movement cost of Eq. 2 and the worked
example around Figures 2 and 3 cannot be replayed (the figures are not available and the
example contradicts the tile-size rule of Algorithm 1): parity unpinned for those two items.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tf_oracle.c")
_LIB = os.path.join(_HERE, "_build", "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile tf_oracle.c with gcc.  -ffp-contract=off keeps multiply and add separate."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
               "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.orc_gemm.argtypes = [i64, i64, i64, vp, vp, vp, vp, i64]
        lib.orc_gemm_ct.argtypes = [i64, i64, i64, vp, vp, vp, vp, i64]
        lib.orc_gemm_ct.restype = None
        lib.orc_spmm.argtypes = [i64, vp, vp, vp, i64, vp, vp, vp, i64]
        lib.orc_gemm_par.argtypes = [i64, i64, i64, vp, vp, vp]
        lib.orc_spmm_par.argtypes = [i64, vp, vp, vp, i64, vp, vp]
        lib.orc_num_threads.restype = ctypes.c_int
        for f in (lib.orc_gemm, lib.orc_spmm, lib.orc_gemm_par, lib.orc_spmm_par):
            f.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def gemm(B, C, rows: Optional[Sequence[int]] = None, out: Optional[np.ndarray] = None,
         parallel: bool = False) -> np.ndarray:
    """D1 = B C in fp64 (k ascending).  With `rows`, only those rows of `out` are written."""
    B = _f64(B)
    C = _f64(C)
    n, bcol = B.shape
    assert C.shape[0] == bcol
    ccol = C.shape[1]
    if out is None:
        out = np.zeros((n, ccol), dtype=np.float64)
    lib = _load()
    if parallel:
        assert rows is None
        lib.orc_gemm_par(n, bcol, ccol, _ptr(B), _ptr(C), _ptr(out))
    else:
        r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
        lib.orc_gemm(n, bcol, ccol, _ptr(B), _ptr(C), _ptr(out), _ptr(r),
                     0 if r is None else r.size)
    return out


def gemm_ct(B, Ct, rows: Optional[Sequence[int]] = None, out: Optional[np.ndarray] = None
            ) -> np.ndarray:
    """D1 = B Ct^T in fp64 (k ascending) for Ct given as cCol x bCol: the first operation of the
    chain with the transpose of C (Section 3.2)."""
    B = _f64(B)
    Ct = _f64(Ct)
    n, bcol = B.shape
    assert Ct.shape[1] == bcol
    ccol = Ct.shape[0]
    if out is None:
        out = np.zeros((n, ccol), dtype=np.float64)
    r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    _load().orc_gemm_ct(n, bcol, ccol, _ptr(B), _ptr(Ct), _ptr(out), _ptr(r),
                        0 if r is None else r.size)
    return out


def chain_ct(A, B, Ct, with_scale: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """D = A (B Ct^T) for a dense B and Ct given as cCol x bCol, and optionally
    W = |A| (|B| |Ct|^T); both fp64, full size."""
    D = spmm(A.rowptr, A.colidx, A.vals, gemm_ct(B, Ct))
    W = None
    if with_scale:
        W1 = gemm_ct(np.abs(_f64(B)), np.abs(_f64(Ct)))
        W = spmm(A.rowptr, A.colidx, np.abs(_f64(A.vals)), W1)
    return D, W


def spmm(rowptr, colidx, vals, X, rows: Optional[Sequence[int]] = None,
         out: Optional[np.ndarray] = None, parallel: bool = False) -> np.ndarray:
    """Y = S X for a CSR matrix S (entries summed in storage order), fp64."""
    rowptr = _i32(rowptr)
    colidx = _i32(colidx)
    vals = _f64(vals)
    X = _f64(X)
    n = rowptr.size - 1
    ccol = X.shape[1]
    if colidx.size:
        assert 0 <= int(colidx.min()) and int(colidx.max()) < X.shape[0]
    if out is None:
        out = np.zeros((n, ccol), dtype=np.float64)
    lib = _load()
    if parallel:
        assert rows is None
        lib.orc_spmm_par(n, _ptr(rowptr), _ptr(colidx), _ptr(vals), ccol, _ptr(X), _ptr(out))
    else:
        r = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
        lib.orc_spmm(n, _ptr(rowptr), _ptr(colidx), _ptr(vals), ccol, _ptr(X), _ptr(out),
                     _ptr(r), 0 if r is None else r.size)
    return out


def _first_op(B, C, parallel: bool, rows=None, out=None) -> np.ndarray:
    """D1 = B C with B dense (ndarray) or CSR (tuple-like with rowptr, colidx, vals)."""
    if isinstance(B, np.ndarray):
        return gemm(B, C, rows=rows, out=out, parallel=parallel)
    return spmm(B.rowptr, B.colidx, B.vals, C, rows=rows, out=out, parallel=parallel)


def _abs_of(M):
    if isinstance(M, np.ndarray):
        return np.abs(_f64(M))
    return type(M)(M.n_rows, M.n_cols, M.rowptr, M.colidx, np.abs(_f64(M.vals)))


def chain(A, B, C, parallel: bool = False, with_scale: bool = True
          ) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """D = A (B C) and, optionally, W = |A| (|B| |C|); both fp64, full size."""
    D1 = _first_op(B, C, parallel)
    D = spmm(A.rowptr, A.colidx, A.vals, D1, parallel=parallel)
    W = None
    if with_scale:
        W1 = _first_op(_abs_of(B), np.abs(_f64(C)), parallel)
        W = spmm(A.rowptr, A.colidx, np.abs(_f64(A.vals)), W1, parallel=parallel)
    return D, W


def chain_rows(A, B, C, rows: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Rows `rows` of D and W only (for full-size problems): the D1 rows those rows of A refer
    to are computed first, then the listed rows of D.  Returns arrays of shape [len(rows), cCol].
    """
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    n = A.n_rows
    ccol = C.shape[1]
    need = np.unique(np.concatenate(
        [A.colidx[A.rowptr[j]:A.rowptr[j + 1]] for j in rows] + [np.zeros(0, np.int32)]
    )).astype(np.int64)
    # compact problem: renumber the needed D1 rows 0..m-1
    remap = {int(g): l for l, g in enumerate(need)}
    sub_ptr = [0]
    sub_col = []
    sub_val = []
    for j in rows:
        lo, hi = int(A.rowptr[j]), int(A.rowptr[j + 1])
        sub_col.extend(remap[int(c)] for c in A.colidx[lo:hi])
        sub_val.append(np.asarray(A.vals[lo:hi], dtype=np.float64))
        sub_ptr.append(len(sub_col))
    sub_val = np.concatenate(sub_val) if sub_val else np.zeros(0)
    out = []
    for absolute in (False, True):
        Cm = np.abs(_f64(C)) if absolute else _f64(C)
        if isinstance(B, np.ndarray):
            Bm = _f64(B[need])
            Bm = np.abs(Bm) if absolute else Bm
            D1 = gemm(Bm, Cm)
        else:
            bp = [0]
            bc = []
            bv = []
            for i in need:
                lo, hi = int(B.rowptr[i]), int(B.rowptr[i + 1])
                bc.append(np.asarray(B.colidx[lo:hi]))
                bv.append(np.asarray(B.vals[lo:hi], dtype=np.float64))
                bp.append(bp[-1] + hi - lo)
            bc = np.concatenate(bc) if bc else np.zeros(0, np.int32)
            bv = np.concatenate(bv) if bv else np.zeros(0)
            bv = np.abs(bv) if absolute else bv
            D1 = spmm(np.asarray(bp), bc, bv, Cm) if need.size else np.zeros((0, ccol))
        v = np.abs(sub_val) if absolute else sub_val
        if need.size == 0:
            D1 = np.zeros((1, ccol))
        out.append(spmm(np.asarray(sub_ptr), np.asarray(sub_col, dtype=np.int32), v, D1))
    assert n >= 0
    return out[0], out[1]


def rowwise_rel_err(D_test: np.ndarray, D_ref: np.ndarray, W: np.ndarray) -> float:
    """max_j  max_c |D_test - D_ref|[j][c] / s_j  with  s_j = max_c W[j][c].
    Rows with s_j = 0 must be exactly zero in D_test (returns inf otherwise)."""
    diff = np.abs(np.asarray(D_test, dtype=np.float64) - D_ref)
    s = W.max(axis=1) if W.size else np.zeros(W.shape[0])
    rowmax = diff.max(axis=1) if diff.size else np.zeros(diff.shape[0])
    zero = s == 0
    if np.any(rowmax[zero] != 0):
        return float("inf")
    if np.all(zero):
        return 0.0
    return float((rowmax[~zero] / s[~zero]).max())


def elementwise_rel_err(D_test: np.ndarray, D_ref: np.ndarray, W: np.ndarray) -> float:
    """max over elements with W > 0 of |D_test - D_ref| / W (the stricter, reported figure)."""
    diff = np.abs(np.asarray(D_test, dtype=np.float64) - D_ref)
    m = W > 0
    if not np.any(m):
        return 0.0
    return float((diff[m] / W[m]).max())
