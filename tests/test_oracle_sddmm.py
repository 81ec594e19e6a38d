"""Pins of the SDDMM oracle (CPU only): the values a hand-worked example
fixes, the definition as a brute-force dense product that is then sampled,
exact integer inputs, special cases with closed forms, and scipy."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2209_02882_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_csr(rng, M, K, density, integer=False):
    mask = rng.random((M, K)) < density
    if M > 2:
        mask[rng.integers(0, M)] = False  # an empty row
    rowptr = np.zeros(M + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(mask.sum(1))
    colidx = np.nonzero(mask)[1].astype(np.int32)
    vals = wl.fill_values(rng, colidx.size, integer)
    return rowptr, colidx, vals


def rows_of(rowptr):
    return np.repeat(np.arange(rowptr.size - 1), np.diff(rowptr))


def brute_force(M, K, J, rowptr, colidx, vals, X1, X2T):
    """The dense product X1 * X2 by a triple loop in Python floats, sampled on A's pattern."""
    X2 = X2T.T  # X2[j, k]
    D = [[sum(float(X1[i, j]) * float(X2[j, k]) for j in range(J)) for k in range(K)] for i in range(M)]
    out = []
    for i in range(M):
        for p in range(rowptr[i], rowptr[i + 1]):
            out.append(float(vals[p]) * D[i][colidx[p]])
    return np.array(out, dtype=np.float64)


def test_golden_hand_worked_example():
    d = {}
    with open(os.path.join(GOLDEN, "sddmm_2x3_by_hand.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = v
    M, K, J = int(d["M"][0]), int(d["K"][0]), int(d["J"][0])
    rowptr = np.array(d["rowptr"], dtype=np.int32)
    colidx = np.array(d["colidx"], dtype=np.int32)
    vals = np.array(d["vals"], dtype=np.float32)
    X1 = np.array(d["X1"], dtype=np.float32).reshape(M, J)
    X2T = np.array(d["X2T"], dtype=np.float32).reshape(K, J)
    out, BND = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T)
    assert np.array_equal(out, np.array(d["out"], dtype=np.float64))
    assert np.array_equal(BND, np.array(d["BND"], dtype=np.float64))


@pytest.mark.parametrize("M,K,J", [(1, 1, 1), (5, 7, 3), (17, 9, 4), (8, 33, 6), (24, 16, 11)])
def test_matches_brute_force_definition(M, K, J):
    # non-square shapes, M != K != J: a swapped operand or index cannot survive
    rng = np.random.default_rng(300 + M * K + J)
    rowptr, colidx, vals = random_csr(rng, M, K, 0.3)
    X1 = wl.fill_values(rng, M * J, False).reshape(M, J)
    X2T = wl.fill_values(rng, K * J, False).reshape(K, J)
    out, BND = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T)
    ref = brute_force(M, K, J, rowptr, colidx, vals, X1, X2T)
    assert out.shape == ref.shape
    assert np.all(np.abs(out - ref) <= 1e-12 * np.maximum(BND, 1e-300))


def test_exact_on_integer_inputs():
    rng = np.random.default_rng(31)
    M, K, J = 30, 40, 9
    rowptr, colidx, vals = random_csr(rng, M, K, 0.25, integer=True)
    X1 = wl.fill_values(rng, M * J, True).reshape(M, J)
    X2T = wl.fill_values(rng, K * J, True).reshape(K, J)
    out, _ = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T)
    ref = brute_force(M, K, J, rowptr, colidx, vals, X1, X2T)
    assert np.array_equal(out, ref)
    assert np.array_equal(out, np.round(out))


def test_closed_forms():
    rng = np.random.default_rng(32)
    M, K, J = 12, 10, 5
    rowptr, colidx, vals = random_csr(rng, M, K, 0.4)
    rows = rows_of(rowptr)
    # all-ones operands: every dot product is J
    out, BND = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, np.ones((M, J)), np.ones((K, J)))
    assert np.array_equal(out, vals.astype(np.float64) * J)
    assert np.array_equal(BND, np.abs(vals.astype(np.float64)) * J)
    # J = 1: a product of three numbers
    x1 = wl.fill_values(rng, M, False).reshape(M, 1)
    x2 = wl.fill_values(rng, K, False).reshape(K, 1)
    out, _ = oracle.sddmm_csr(M, K, 1, rowptr, colidx, vals, x1, x2)
    assert np.array_equal(out, vals.astype(np.float64) * (x1[rows, 0].astype(np.float64) * x2[colidx, 0].astype(np.float64)))
    # X2 = identity (J = K): the entry picks X1[i, k]
    X1 = wl.fill_values(rng, M * K, False).reshape(M, K)
    out, _ = oracle.sddmm_csr(M, K, K, rowptr, colidx, vals, X1, np.eye(K, dtype=np.float32))
    assert np.array_equal(out, vals.astype(np.float64) * X1[rows, colidx].astype(np.float64))
    # J = 0: empty sums
    out, BND = oracle.sddmm_csr(M, K, 0, rowptr, colidx, vals, np.zeros((M, 0)), np.zeros((K, 0)))
    assert np.all(out == 0) and np.all(BND == 0)


def test_row_scaling_and_linearity():
    rng = np.random.default_rng(33)
    M, K, J = 9, 14, 6
    rowptr, colidx, vals = random_csr(rng, M, K, 0.35, integer=True)
    X1 = wl.fill_values(rng, M * J, True).reshape(M, J)
    X2T = wl.fill_values(rng, K * J, True).reshape(K, J)
    base, _ = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T)
    rows = rows_of(rowptr)
    # scaling row 3 of X1 scales exactly the entries of row 3
    X1s = X1.copy()
    X1s[3] *= 2
    out, _ = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1s, X2T)
    assert np.array_equal(out, np.where(rows == 3, 2 * base, base))
    # scaling row 5 of X2T scales exactly the entries in column 5
    X2s = X2T.copy()
    X2s[5] *= -2
    out, _ = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2s)
    assert np.array_equal(out, np.where(colidx == 5, -2 * base, base))
    # additive in X1
    X1b = wl.fill_values(rng, M * J, True).reshape(M, J)
    o2, _ = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1b, X2T)
    o3, _ = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1 + X1b, X2T)
    assert np.array_equal(o3, base + o2)


def test_matches_scipy_sampled_product():
    rng = np.random.default_rng(34)
    M, K, J = 60, 45, 17
    rowptr, colidx, vals = random_csr(rng, M, K, 0.2)
    X1 = wl.fill_values(rng, M * J, False).reshape(M, J)
    X2T = wl.fill_values(rng, K * J, False).reshape(K, J)
    out, BND = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T)
    A = sp.csr_matrix((vals.astype(np.float64), colidx, rowptr), shape=(M, K))
    ref = A.multiply(X1.astype(np.float64) @ X2T.astype(np.float64).T).tocsr()
    dense = ref.toarray()
    assert np.all(np.abs(out - dense[rows_of(rowptr), colidx]) <= 1e-12 * np.maximum(BND, 1e-300))


def test_threads_agree_and_duplicates_are_separate_entries():
    rng = np.random.default_rng(35)
    M, K, J = 50, 20, 8
    rowptr, colidx, vals = random_csr(rng, M, K, 0.3)
    X1 = wl.fill_values(rng, M * J, False).reshape(M, J)
    X2T = wl.fill_values(rng, K * J, False).reshape(K, J)
    o1, b1 = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T, nthreads=1)
    o4, b4 = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T, nthreads=4)
    assert np.array_equal(o1, o4) and np.array_equal(b1, b4)
    # a duplicated, unsorted column index is just another stored entry
    rp = np.array([0, 3], dtype=np.int32)
    ci = np.array([2, 0, 2], dtype=np.int32)
    va = np.array([1.0, 2.0, 3.0], dtype=np.float32)
    out, _ = oracle.sddmm_csr(1, 3, 2, rp, ci, va, np.array([[1.0, 2.0]]), np.array([[1, 1], [5, 5], [2, -1]], dtype=np.float32))
    assert np.array_equal(out, [0.0, 6.0, 0.0])
