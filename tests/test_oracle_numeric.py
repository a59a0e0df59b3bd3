"""Pins of the numeric CPU oracle against things other than itself (no GPU needed).

Each test is chosen so that a plausible mistake in oracle/tf_oracle.c -- a dropped term, a
transposed operand, a wrong index, accumulate-instead-of-overwrite -- fails at least one.
"""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import tf_inputs as ti

U64 = 2.0 ** -53


def gamma(k):
    return k * U64 / (1 - k * U64)


def dense_of(A):
    """Dense matrix of a CSR with duplicates summed (python loops: tiny inputs only)."""
    M = np.zeros((A.n_rows, A.n_cols), dtype=np.longdouble)
    for j in range(A.n_rows):
        for q in range(A.rowptr[j], A.rowptr[j + 1]):
            M[j, A.colidx[q]] += np.longdouble(A.vals[q])
    return M


def brute_force_chain(A, B, C):
    """D[j][c] = sum_i sum_k A[j][i] B[i][k] C[k][c] in extended precision, pure loops."""
    Ad = dense_of(A)
    Bd = dense_of(B) if isinstance(B, ti.Csr) else B.astype(np.longdouble)
    Cd = C.astype(np.longdouble)
    n, m = Ad.shape[0], Cd.shape[1]
    D = np.zeros((n, m), dtype=np.longdouble)
    for j in range(n):
        for i in range(Ad.shape[1]):
            a = Ad[j, i]
            if a == 0:
                continue
            for k in range(Bd.shape[1]):
                b = Bd[i, k]
                if b == 0:
                    continue
                for c in range(m):
                    D[j, c] += a * b * Cd[k, c]
    return D


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_brute_force_dense_b(seed, dtype):
    n, bcol, ccol = 13, 5, 7          # non-square on purpose: a transposed operand cannot pass
    A = ti.random_pattern_csr(n, n, 0.3, dtype, seed, sort_cols=False, duplicates=True,
                              empty_row_prob=0.2)
    B = ti.dense_normal(n, bcol, dtype, seed + 10)
    C = ti.dense_normal(bcol, ccol, dtype, seed + 20)
    D, W = oracle.chain(A, B, C)
    ref = brute_force_chain(A, B, C)
    k = bcol + int(np.diff(A.rowptr).max())
    assert np.all(np.abs(D - ref.astype(np.float64)) <= 2 * gamma(k) * W + 1e-300)
    # the normaliser itself: brute force on absolute values
    Aa = ti.Csr(A.n_rows, A.n_cols, A.rowptr, A.colidx, np.abs(A.vals))
    refw = brute_force_chain(Aa, np.abs(B), np.abs(C)).astype(np.float64)
    assert np.allclose(W, refw, rtol=1e-13, atol=0)
    # empty rows are written as exact zeros
    empty = np.diff(A.rowptr) == 0
    assert empty.any() and np.all(D[empty] == 0)


@pytest.mark.parametrize("seed", [4, 5])
def test_brute_force_sparse_b(seed):
    n, m, ccol = 11, 9, 6             # B is n x m, C is m x ccol
    A = ti.random_pattern_csr(n, n, 0.35, np.float64, seed, sort_cols=False, duplicates=True,
                              empty_row_prob=0.15)
    B = ti.random_pattern_csr(n, m, 0.4, np.float64, seed + 1, sort_cols=False,
                              duplicates=True, empty_row_prob=0.1)
    C = ti.dense_normal(m, ccol, np.float64, seed + 2)
    D, W = oracle.chain(A, B, C)
    ref = brute_force_chain(A, B, C).astype(np.float64)
    k = int(np.diff(A.rowptr).max()) + int(np.diff(B.rowptr).max())
    assert np.all(np.abs(D - ref) <= 2 * gamma(k) * W + 1e-300)


def identity_csr(n, dtype):
    return ti.Csr(n, n, np.arange(n + 1, dtype=np.int32), np.arange(n, dtype=np.int32),
                  np.ones(n, dtype=dtype))


def test_identity_a_gives_bc_bitwise():
    n, bcol, ccol = 40, 16, 24
    B = ti.dense_normal(n, bcol, np.float64, 7)
    C = ti.dense_normal(bcol, ccol, np.float64, 8)
    D, _ = oracle.chain(identity_csr(n, np.float64), B, C)
    D1 = oracle.gemm(B, C)
    assert np.array_equal(D, D1)
    # and D1 is B C: against the library matmul, within the textbook bound
    W1 = np.abs(B) @ np.abs(C)
    assert np.all(np.abs(D1 - B @ C) <= 2 * gamma(bcol) * W1)


def test_identity_b_gives_ac_bitwise():
    n, ccol = 30, 8
    A = ti.random_pattern_csr(n, n, 0.2, np.float64, 11, sort_cols=True)
    C = ti.dense_normal(n, ccol, np.float64, 12)
    D, _ = oracle.chain(A, identity_csr(n, np.float64), C)
    assert np.array_equal(D, oracle.spmm(A.rowptr, A.colidx, A.vals, C))
    ref = sp.csr_matrix((A.vals, A.colidx, A.rowptr), shape=(n, n)) @ C
    assert np.allclose(D, ref, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("kind", ["dense", "sparse"])
def test_associativity(kind):
    n, bcol, ccol = 24, 10, 12
    A = ti.random_pattern_csr(n, n, 0.25, np.float64, 21)
    As = sp.csr_matrix((A.vals, A.colidx, A.rowptr), shape=(n, n))
    if kind == "dense":
        B = ti.dense_normal(n, bcol, np.float64, 22)
        AB = As @ B
        absAB = abs(As) @ np.abs(B)
    else:
        B = ti.random_pattern_csr(n, bcol, 0.4, np.float64, 22)
        Bs = sp.csr_matrix((B.vals, B.colidx, B.rowptr), shape=(n, bcol))
        AB = (As @ Bs).toarray()
        absAB = (abs(As) @ abs(Bs)).toarray()
    C = ti.dense_normal(bcol, ccol, np.float64, 23)
    D, W = oracle.chain(A, B, C)
    left = AB @ C                      # (AB)C
    bound = 4 * gamma(n + bcol) * (absAB @ np.abs(C))
    assert np.all(np.abs(D - left) <= bound + 1e-300)
    assert np.allclose(W, absAB @ np.abs(C), rtol=1e-12)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("kind", ["dense", "sparse"])
def test_small_integers_are_exact(dtype, kind):
    """Entries in {-2..2}: every partial sum is a small integer, so any summation order is exact
    and the oracle must equal integer arithmetic bit for bit."""
    n, bcol, ccol = 50, 12, 9
    A = ti.random_pattern_csr(n, n, 0.2, dtype, 31, sort_cols=False, duplicates=True,
                              empty_row_prob=0.1, int_values=True)
    C = ti.dense_small_int(bcol, ccol, dtype, 33)
    Ai = np.zeros((n, n), dtype=np.int64)
    for j in range(n):
        for q in range(A.rowptr[j], A.rowptr[j + 1]):
            Ai[j, A.colidx[q]] += int(A.vals[q])
    if kind == "dense":
        B = ti.dense_small_int(n, bcol, dtype, 32)
        Bi = B.astype(np.int64)
    else:
        B = ti.random_pattern_csr(n, bcol, 0.3, dtype, 32, int_values=True, duplicates=True)
        Bi = np.zeros((n, bcol), dtype=np.int64)
        for j in range(n):
            for q in range(B.rowptr[j], B.rowptr[j + 1]):
                Bi[j, B.colidx[q]] += int(B.vals[q])
    D, _ = oracle.chain(A, B, C)
    expect = Ai @ (Bi @ C.astype(np.int64))
    assert np.array_equal(D, expect.astype(np.float64))


def test_banded_all_ones_counts_row_lengths():
    n, h, ccol = 64, 3, 5
    A = ti.banded(n, h, np.float64, 0, ones=True)
    D1 = np.ones((n, ccol))
    D = oracle.spmm(A.rowptr, A.colidx, A.vals, D1)
    lens = np.diff(A.rowptr).astype(np.float64)
    assert A.nnz == (2 * h + 1) * n - h * (h + 1)
    assert np.array_equal(D, np.repeat(lens[:, None], ccol, axis=1))


def test_banded_nnz_of_config1():
    assert ti.banded(4096, 8, np.float64, 1).nnz == 17 * 4096 - 72


def test_laplacian_closed_forms():
    g = 6
    L2 = ti.laplacian_2d(g, np.float64)
    assert L2.nnz == 5 * g * g - 4 * g
    D = oracle.spmm(L2.rowptr, L2.colidx, L2.vals, np.ones((g * g, 3)))
    x = np.arange(g * g) % g
    y = np.arange(g * g) // g
    missing = (x == 0).astype(int) + (x == g - 1) + (y == 0) + (y == g - 1)
    assert np.array_equal(D[:, 0], missing.astype(np.float64))     # 4 - #neighbours
    L3 = ti.laplacian_3d(g, np.float64)
    assert L3.nnz == 7 * g ** 3 - 6 * g * g
    D = oracle.spmm(L3.rowptr, L3.colidx, L3.vals, np.ones((g ** 3, 2)))
    i = np.arange(g ** 3)
    x, y, z = i % g, (i // g) % g, i // (g * g)
    missing = sum(((v == 0).astype(int) + (v == g - 1)) for v in (x, y, z))
    assert np.array_equal(D[:, 1], missing.astype(np.float64))
    # full chain with B = the same Laplacian: L (L 1) = L * missing, against scipy
    Ls = sp.csr_matrix((L3.vals, L3.colidx, L3.rowptr), shape=(g ** 3,) * 2)
    Dc, _ = oracle.chain(L3, L3, np.ones((g ** 3, 2)))
    assert np.array_equal(Dc[:, 0], Ls @ missing.astype(np.float64))


def test_gcn_eigenvector():
    """deg^-1/2 (Adj+I) deg^-1/2 has eigenvalue 1 with eigenvector deg^1/2."""
    s = 8
    A = ti.gcn_normalised(s, 8 << s, np.float64, 5)
    n = 1 << s
    As = sp.csr_matrix((A.vals, A.colidx, A.rowptr), shape=(n, n))
    assert abs(As - As.T).max() < 1e-15
    deg = np.zeros(n)
    np.add.at(deg, np.repeat(np.arange(n), np.diff(A.rowptr)), 1.0)
    v = np.sqrt(deg)
    D1 = np.repeat(v[:, None], 4, axis=1)
    D = oracle.spmm(A.rowptr, A.colidx, A.vals, D1)
    assert np.allclose(D, D1, rtol=1e-13, atol=0)


def test_against_scipy_on_structured_cases():
    """Special cases that reduce to library routines: scipy CSR @ (numpy matmul)."""
    for cfg, sd in ((1, 300), (2, 12), (4, 6), (3, 8), (5, 8)):
        p = ti.config(cfg, scale_down=sd)
        D, W = oracle.chain(p.A, p.B, p.C)
        As = sp.csr_matrix((p.A.vals.astype(np.float64), p.A.colidx, p.A.rowptr),
                           shape=(p.n, p.n))
        if p.kind == "gemm_spmm":
            D1 = p.B.astype(np.float64) @ p.C.astype(np.float64)
        else:
            Bs = sp.csr_matrix((p.B.vals.astype(np.float64), p.B.colidx, p.B.rowptr),
                               shape=(p.B.n_rows, p.B.n_cols))
            D1 = Bs @ p.C.astype(np.float64)
        ref = As @ D1
        assert oracle.rowwise_rel_err(ref, D, W) < 1e-13
        assert oracle.elementwise_rel_err(ref, D, W) < 1e-13


def test_overwrite_not_accumulate():
    p = ti.config(1, scale_down=64)
    out = np.full((p.n, p.ccol), 123.0)
    D1 = oracle.gemm(p.B, p.C, out=out)
    assert np.array_equal(D1, oracle.gemm(p.B, p.C))


def test_parallel_is_bit_identical():
    for cfg, sd in ((2, 20), (5, 9)):
        p = ti.config(cfg, scale_down=sd)
        D, W = oracle.chain(p.A, p.B, p.C)
        Dp, Wp = oracle.chain(p.A, p.B, p.C, parallel=True)
        assert np.array_equal(D, Dp) and np.array_equal(W, Wp)


def test_chain_rows_matches_full():
    for cfg, sd in ((3, 9), (4, 7)):
        p = ti.config(cfg, scale_down=sd)
        D, W = oracle.chain(p.A, p.B, p.C)
        rows = np.array([0, 1, p.n // 2, p.n - 1, 5, 5])
        Dr, Wr = oracle.chain_rows(p.A, p.B, p.C, rows)
        assert np.array_equal(Dr, D[rows]) and np.array_equal(Wr, W[rows])


def test_error_metric_flags_nonzero_in_empty_row():
    D = np.zeros((3, 2))
    W = np.array([[1.0, 2.0], [0.0, 0.0], [3.0, 1.0]])
    T = D.copy()
    assert oracle.rowwise_rel_err(T, D, W) == 0.0
    T[1, 0] = 1e-30
    assert oracle.rowwise_rel_err(T, D, W) == float("inf")
    T[1, 0] = 0
    T[2, 1] = 3e-6
    assert abs(oracle.rowwise_rel_err(T, D, W) - 1e-6) < 1e-18
    assert abs(oracle.elementwise_rel_err(T, D, W) - 3e-6) < 1e-18


# ---- the chain with the transpose of C (Section 3.2)

def test_transposed_c_hand_worked():
    """B = [1 2], Ct = [[3 4], [5 6]]: B Ct^T = [1*3 + 2*4, 1*5 + 2*6] = [11 17], whereas the
    plain product B Ct = [13 16]; a transposed index gives the other one."""
    B = np.array([[1.0, 2.0]])
    Ct = np.array([[3.0, 4.0], [5.0, 6.0]])
    assert np.array_equal(oracle.gemm_ct(B, Ct), [[11.0, 17.0]])
    assert np.array_equal(oracle.gemm(B, Ct), [[13.0, 16.0]])


@pytest.mark.parametrize("seed", [1, 2])
def test_transposed_c_brute_force(seed):
    n, bcol, ccol = 11, 5, 7          # non-square: a wrong stride reads the wrong element
    A = ti.random_pattern_csr(n, n, 0.3, np.float64, seed, sort_cols=False, duplicates=True,
                              empty_row_prob=0.2)
    B = ti.dense_normal(n, bcol, np.float64, seed + 10)
    Ct = ti.dense_normal(ccol, bcol, np.float64, seed + 20)
    D, W = oracle.chain_ct(A, B, Ct)
    ref = brute_force_chain(A, B, np.ascontiguousarray(Ct.T))
    k = bcol + int(np.diff(A.rowptr).max())
    assert np.all(np.abs(D - ref.astype(np.float64)) <= 2 * gamma(k) * W + 1e-300)
    # same summation order as the plain chain on the explicitly transposed array: bit-identical
    D2, W2 = oracle.chain(A, B, np.ascontiguousarray(Ct.T))
    assert np.array_equal(D, D2) and np.array_equal(W, W2)
    # listed rows only: the others stay untouched
    out = np.full((n, ccol), 7.0)
    oracle.gemm_ct(B, Ct, rows=[2, 5], out=out)
    full = oracle.gemm_ct(B, Ct)
    assert np.array_equal(out[[2, 5]], full[[2, 5]]) and np.all(np.delete(out, [2, 5], 0) == 7.0)
