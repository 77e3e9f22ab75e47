"""Pins for the CPU oracle (fp64 CSR SpMM, Section 2 problem statement / Algorithm 1 loop).

Each pin is something other than the oracle's own formula: a dense matmul, closed forms,
a hand-worked example, invariants, a library routine, brute force from the definition.
"""
import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import synth
from tests.helpers import dense_to_csr, random_csr


def test_hand_worked_example():
    # A = [[2, 0, -1], [0, 0, 0], [0.5, 3, 0]],  B = [[1, 2], [3, 4], [5, 6]]
    # A @ B = [[2-5, 4-6], [0, 0], [0.5+9, 1+12]] = [[-3, -2], [0, 0], [9.5, 13]]
    rowptr = np.array([0, 2, 2, 4], np.int32)
    colidx = np.array([0, 2, 0, 1], np.int32)
    vals = np.array([2, -1, 0.5, 3], np.float32)
    B = np.array([[1, 2], [3, 4], [5, 6]], np.float32)
    C, bound = oracle.spmm(rowptr, colidx, vals, B)
    assert np.array_equal(C, np.array([[-3, -2], [0, 0], [9.5, 13]], np.float64))
    # sum |a*b|: [[2+5, 4+6], [0, 0], [0.5+9, 1+12]]
    assert np.array_equal(bound, np.array([[7, 10], [0, 0], [9.5, 13]], np.float64))


@pytest.mark.parametrize("n,density,K", [(1, 1.0, 1), (7, 0.3, 5), (33, 0.1, 16), (64, 0.5, 37),
                                         (50, 0.02, 8)])
def test_against_dense_matmul(n, density, K):
    rng = np.random.default_rng(100 + n)
    rowptr, colidx, vals, dense = random_csr(rng, n, n, density, empty_rows=(0,) if n > 2 else (),
                                             full_rows=(n - 1,) if n > 2 else ())
    B = rng.standard_normal((n, K)).astype(np.float32)
    C, bound = oracle.spmm(rowptr, colidx, vals, B)
    ref = dense.astype(np.float64) @ B.astype(np.float64)
    refb = np.abs(dense.astype(np.float64)) @ np.abs(B.astype(np.float64))
    assert np.allclose(C, ref, rtol=1e-13, atol=1e-13)
    assert np.allclose(bound, refb, rtol=1e-13, atol=1e-13)
    # a non-symmetric A would expose a transposed operand
    assert not np.allclose(dense, dense.T) or n == 1


def test_rectangular_against_dense():
    rng = np.random.default_rng(5)
    rowptr, colidx, vals, dense = random_csr(rng, 9, 23, 0.2)
    B = rng.standard_normal((23, 6)).astype(np.float32)
    C, _ = oracle.spmm(rowptr, colidx, vals, B)
    assert np.allclose(C, dense.astype(np.float64) @ B.astype(np.float64), rtol=1e-13, atol=1e-13)


def test_brute_force_definition():
    rng = np.random.default_rng(7)
    rowptr, colidx, vals, _ = random_csr(rng, 11, 11, 0.3, empty_rows=(4,))
    K = 3
    B = rng.uniform(-1, 1, (11, K)).astype(np.float32)
    C, bound = oracle.spmm(rowptr, colidx, vals, B)
    for i in range(11):
        for k in range(K):
            s, sb = 0.0, 0.0
            for p in range(rowptr[i], rowptr[i + 1]):
                t = float(vals[p]) * float(B[colidx[p], k])
                s += t
                sb += abs(t)
            assert C[i, k] == s and bound[i, k] == sb


def test_identity_gives_B_bit_exact():
    n, K = 40, 12
    rowptr = np.arange(n + 1, dtype=np.int32)
    colidx = np.arange(n, dtype=np.int32)
    vals = np.ones(n, np.float32)
    B = np.random.default_rng(1).standard_normal((n, K)).astype(np.float32)
    C, _ = oracle.spmm(rowptr, colidx, vals, B)
    assert np.array_equal(C.astype(np.float32).view(np.uint32), B.view(np.uint32))


def test_permutation_matrix_moves_rows():
    n, K = 31, 4
    perm = np.random.default_rng(2).permutation(n).astype(np.int32)
    B = np.random.default_rng(3).standard_normal((n, K)).astype(np.float32)
    C, _ = oracle.spmm(np.arange(n + 1, dtype=np.int32), perm, np.ones(n, np.float32), B)
    assert np.array_equal(C, B[perm].astype(np.float64))


@pytest.mark.parametrize("name", ["poisson", "sbm"])
def test_all_ones_B_mean_aggregation_rows_sum_to_one(name):
    g = synth.workload(name, "small")
    B = np.ones((g.n_cols, 4), np.float32)
    C, bound = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    deg = g.degrees()
    assert np.all(C[deg == 0] == 0.0)
    # vals = fp32(1/deg): the row sum is deg * fp32(1/deg), within fp32 rounding of 1
    assert np.allclose(C[deg > 0], 1.0, rtol=0, atol=1e-7)
    assert np.array_equal(C, bound)          # all terms positive
    assert np.all(C == C[:, :1])             # every column identical


def test_all_ones_B_gives_weighted_row_sums():
    g = synth.workload("road", "small")
    C, _ = oracle.spmm(g.rowptr, g.colidx, g.vals, np.ones((g.n_cols, 3), np.float32))
    rowsum = np.add.reduceat(np.concatenate([g.vals.astype(np.float64), [0.0]]),
                             np.minimum(g.rowptr[:-1], g.nnz))
    rowsum[g.degrees() == 0] = 0.0
    assert np.allclose(C[:, 0], rowsum, rtol=1e-14, atol=0)


def test_permutation_invariance_under_relabelling():
    g = synth.workload("rmat20", "small")
    n, K = g.n_rows, 8
    B = synth.dense_operand(n, K, "normal", 11)
    C, _ = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    pi = np.random.default_rng(9).permutation(n)      # new id of old node i is pi[i]
    A = sp.csr_matrix((g.vals, g.colidx, g.rowptr), shape=(n, n)).tocoo()
    A2 = sp.csr_matrix((A.data, (pi[A.row], pi[A.col])), shape=(n, n))
    A2.sort_indices()
    B2 = np.empty_like(B)
    B2[pi] = B
    C2, _ = oracle.spmm(A2.indptr.astype(np.int32), A2.indices.astype(np.int32), A2.data, B2)
    assert np.allclose(C2[pi], C, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("name,K", [("rmat20", 16), ("sbm_shuffled", 8), ("road", 32)])
def test_scipy_cross_check(name, K):
    g = synth.workload(name, "small")
    B = synth.dense_operand(g.n_cols, K, "normal", 3)
    C, bound = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    A = sp.csr_matrix((g.vals.astype(np.float64), g.colidx, g.rowptr), shape=(g.n_rows, g.n_cols))
    ref = A @ B.astype(np.float64)
    assert np.allclose(C, ref, rtol=1e-12, atol=1e-14)
    assert np.all(bound >= np.abs(C) - 1e-15)
    refb = abs(A) @ np.abs(B.astype(np.float64))
    assert np.allclose(bound, refb, rtol=1e-12, atol=1e-14)


def test_selected_rows_match_full_product_and_threads_do_not_matter():
    g = synth.workload("rmat20", "small")
    B = synth.dense_operand(g.n_cols, 8, "normal", 4)
    C, bound = oracle.spmm(g.rowptr, g.colidx, g.vals, B)
    C1, bound1 = oracle.spmm(g.rowptr, g.colidx, g.vals, B, n_threads=1)
    assert np.array_equal(C, C1) and np.array_equal(bound, bound1)
    rows = np.array([0, 5, g.n_rows - 1, int(np.argmax(g.degrees()))], np.int64)
    Cs, bs = oracle.spmm_rows(g.rowptr, g.colidx, g.vals, B, rows)
    assert np.array_equal(Cs, C[rows]) and np.array_equal(bs, bound[rows])


def test_empty_matrix_and_zero_K():
    C, bound = oracle.spmm(np.zeros(5, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                           np.ones((4, 3), np.float32))
    assert C.shape == (4, 3) and not C.any() and not bound.any()


def test_tolerance_helper():
    ref = np.array([[1.0, 2.0]])
    bound = np.array([[1.0, 2.0]])
    ok, _ = oracle.within_tolerance(ref + 5e-6, ref, bound)
    assert ok
    ok, _ = oracle.within_tolerance(ref + np.array([[2e-5, 0]]), ref, bound)
    assert not ok
    ok, _ = oracle.within_tolerance(np.array([[np.nan, 2.0]]), ref, bound)
    assert not ok
