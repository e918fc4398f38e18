"""Pins for the oracle's SpMM (C = A.B, Section 3.1) against things other than
itself: brute-force loops, exact special cases, a library routine."""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2504_06443_amd import workloads as W


def brute_force(A: W.CSR, B: np.ndarray):
    """Dense triple loop in Python floats (fp64), no library product."""
    M, K, N = A.M, A.K, B.shape[1]
    dense = [[0.0] * K for _ in range(M)]
    for i in range(M):
        for e in range(A.rowptr[i], A.rowptr[i + 1]):
            dense[i][int(A.colind[e])] = float(A.vals[e])
    Cb = np.zeros((M, N))
    Sb = np.zeros((M, N))
    for i in range(M):
        for j in range(N):
            acc = 0.0
            sab = 0.0
            for k in range(K):
                p = dense[i][k] * float(B[k, j])
                acc += p
                sab += abs(p)
            Cb[i, j] = acc
            Sb[i, j] = sab
    return Cb, Sb


@pytest.mark.parametrize("M,K,N,density,seed", [
    (1, 1, 1, 1.0, 0), (16, 4, 1, 1.0, 1), (17, 9, 3, 0.4, 2), (33, 50, 8, 0.15, 3),
    (64, 64, 5, 0.05, 4), (40, 7, 2, 0.5, 5), (5, 64, 7, 0.3, 6),
])
def test_matches_dense_brute_force(M, K, N, density, seed):
    A = W.uniform_random(M, K, density, seed, empty_row_frac=0.2 if M > 8 else 0.0)
    B = W.dense_b(K, N, seed + 100)
    Cb, Sb = brute_force(A, B)
    Co, So = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    # both are fp64 sums of the same fp64 products; order differs only by skipped zeros
    np.testing.assert_allclose(Co, Cb, rtol=0, atol=1e-13 * max(1.0, Sb.max()))
    np.testing.assert_allclose(So, Sb, rtol=1e-14, atol=0)


def test_transposed_operand_would_fail():
    """Non-square A with a non-symmetric pattern: guards against using A^T or B^T."""
    A = W.csr_from_coo(3, 5, [0, 0, 2], [1, 4, 0], np.array([2.0, -3.0, 5.0], np.float32))
    B = np.arange(10, dtype=np.float32).reshape(5, 2) + 1
    Co = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)
    expect = np.array([[2 * 3 - 3 * 9, 2 * 4 - 3 * 10], [0, 0], [5 * 1, 5 * 2]], dtype=np.float64)
    assert np.array_equal(Co, expect)


def test_identity_returns_b_exactly():
    n, N = 100, 7
    A = W.csr_from_coo(n, n, np.arange(n), np.arange(n), np.ones(n, np.float32))
    B = W.dense_b(n, N, 7)
    Co, So = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    assert np.array_equal(Co, B.astype(np.float64))
    assert np.array_equal(So, np.abs(B.astype(np.float64)))


def test_permutation_permutes_rows_exactly():
    n, N = 77, 5
    perm = np.random.default_rng(3).permutation(n)
    A = W.csr_from_coo(n, n, np.arange(n), perm, np.ones(n, np.float32))
    B = W.dense_b(n, N, 8)
    Co = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)
    assert np.array_equal(Co, B[perm].astype(np.float64))


def test_ones_column_gives_row_sums():
    A = W.uniform_random(50, 40, 0.2, 11, integer_values=True)
    B = np.ones((40, 1), dtype=np.float32)
    Co = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)
    rs = np.array([A.vals[A.rowptr[i]:A.rowptr[i + 1]].astype(np.float64).sum() for i in range(50)])
    assert np.array_equal(Co[:, 0], rs)


def test_linearity_in_b():
    A = W.uniform_random(48, 31, 0.2, 12)
    B1, B2 = W.dense_b(31, 6, 1), W.dense_b(31, 6, 2)
    # integer-valued combination keeps fp32 inputs exact
    B3 = (2 * B1.astype(np.float64) - 3 * B2.astype(np.float64))
    B3f = B3.astype(np.float32)
    C1 = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B1, want_abs=False)
    C2 = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B2, want_abs=False)
    C3 = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B3f, want_abs=False)
    lhs = 2 * C1 - 3 * C2
    # B3f is B3 rounded to fp32: allow that rounding, nothing more
    np.testing.assert_allclose(C3, lhs, rtol=0, atol=2e-6 * np.abs(lhs).max())


@pytest.mark.parametrize("maker", [
    lambda: W.tiny_banded(M=512, seed=5),
    lambda: W.clustered_blocks(700, 4, 40, seed=6),
    lambda: W.brick_sweep(0.4, M=256, target_nnz=4000, seed=7),
])
def test_matches_scipy_float64(maker):
    A = maker()
    B = W.dense_b(A.K, 9, 21)
    S = sp.csr_matrix((A.vals.astype(np.float64), A.colind, A.rowptr), shape=(A.M, A.K))
    ref = S @ B.astype(np.float64)
    Co, So = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    np.testing.assert_allclose(Co, ref, rtol=0, atol=1e-13 * So.max())
    refS = abs(S) @ np.abs(B.astype(np.float64))
    np.testing.assert_allclose(So, refS, rtol=1e-13)


def test_sampled_rows_match_brute_force():
    A = W.uniform_random(40, 30, 0.2, 31, empty_row_frac=0.1)
    B = W.dense_b(30, 4, 32)
    Cb, Sb = brute_force(A, B)
    rows = np.array([39, 0, 17, 17, 5])
    Cr, Sr = oracle.spmm_rows_f64(rows, A.rowptr, A.colind, A.vals, B)
    np.testing.assert_allclose(Cr, Cb[rows], rtol=0, atol=1e-13 * max(1.0, Sb.max()))
    np.testing.assert_allclose(Sr, Sb[rows], rtol=1e-14)


def test_empty_cases():
    # M = 0
    Co, So = oracle.spmm_f64(np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                             np.zeros((3, 2), np.float32))
    assert Co.shape == (0, 2)
    # no stored entries: C is all zeros
    Co, So = oracle.spmm_f64(np.zeros(6, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                             np.ones((3, 2), np.float32))
    assert not Co.any() and not So.any()
