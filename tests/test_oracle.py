"""Pins for the CPU oracle (CPU only).  Each test fixes the oracle against
something other than itself: the definition written as a brute-force loop, a
hand-worked example, closed-form special cases, exact integer arithmetic and
an independent library routine."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2209_02882_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_csr(rng, M, K, density, integer=False, empty_rows=True):
    mask = rng.random((M, K)) < density
    if empty_rows and M > 2:
        mask[rng.integers(0, M)] = False
    rowptr = np.zeros(M + 1, dtype=np.int32)
    rowptr[1:] = np.cumsum(mask.sum(1))
    colidx = np.nonzero(mask)[1].astype(np.int32)
    vals = wl.fill_values(rng, colidx.size, integer)
    return rowptr, colidx, vals


def densify(M, K, rowptr, colidx, vals):
    A = np.zeros((M, K), dtype=np.float64)
    for i in range(M):
        for p in range(rowptr[i], rowptr[i + 1]):
            A[i, colidx[p]] += float(vals[p])
    return A


def brute_force(M, K, N, rowptr, colidx, vals, B):
    """The definition as a dense triple loop in Python floats (fp64)."""
    A = densify(M, K, rowptr, colidx, vals)
    C = [[0.0] * N for _ in range(M)]
    for i in range(M):
        for k in range(N):
            s = 0.0
            for j in range(K):
                s += A[i, j] * float(B[j, k])
            C[i][k] = s
    return np.array(C, dtype=np.float64).reshape(M, N)


def test_golden_hand_worked_example():
    d = {}
    with open(os.path.join(GOLDEN, "spmm_3x4_by_hand.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = v
    M, K, N = int(d["M"][0]), int(d["K"][0]), int(d["N"][0])
    rowptr = np.array(d["rowptr"], dtype=np.int32)
    colidx = np.array(d["colidx"], dtype=np.int32)
    vals = np.array(d["vals"], dtype=np.float32)
    B = np.array(d["B"], dtype=np.float32).reshape(K, N)
    C, BND = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, B)
    assert np.array_equal(C, np.array(d["C"], dtype=np.float64).reshape(M, N))
    assert np.array_equal(BND, np.array(d["BND"], dtype=np.float64).reshape(M, N))


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (5, 7, 3), (17, 9, 4), (8, 33, 6), (40, 64, 5)])
def test_matches_brute_force_definition(M, K, N):
    # non-square shapes and unsymmetric values: a transposed operand, a wrong
    # index or a dropped term cannot survive this
    rng = np.random.default_rng(100 + M * K + N)
    rowptr, colidx, vals = random_csr(rng, M, K, 0.3)
    B = wl.fill_values(rng, K * N, False).reshape(K, N)
    C, BND = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, B)
    ref = brute_force(M, K, N, rowptr, colidx, vals, B)
    scale = np.abs(densify(M, K, rowptr, colidx, vals)) @ np.abs(B.astype(np.float64))
    assert np.all(np.abs(C - ref) <= 1e-12 * scale + 1e-300)
    assert np.allclose(BND, scale, rtol=1e-12, atol=0)


def test_integer_inputs_are_exact():
    # values in {-2..2}: every product and partial sum is a small integer, so
    # any precision and any order of summation gives the same number
    rng = np.random.default_rng(7)
    M, K, N = 33, 47, 8
    rowptr, colidx, vals = random_csr(rng, M, K, 0.4, integer=True)
    B = wl.fill_values(rng, K * N, True).reshape(K, N)
    C, _ = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, B)
    ref = brute_force(M, K, N, rowptr, colidx, vals, B)
    assert np.array_equal(C, ref)
    assert np.array_equal(C, np.rint(C))
    assert np.array_equal(C.astype(np.float32).astype(np.float64), C)


def test_empty_matrix_gives_zero():
    M, K, N = 9, 5, 4
    rowptr = np.zeros(M + 1, dtype=np.int32)
    B = np.full((K, N), np.float32(3.5))
    C, BND = oracle.spmm_csr(M, K, N, rowptr, np.zeros(0, np.int32), np.zeros(0, np.float32), B)
    assert np.array_equal(C, np.zeros((M, N)))
    assert np.array_equal(BND, np.zeros((M, N)))


def test_identity_returns_B_bit_for_bit():
    rng = np.random.default_rng(3)
    K, N = 29, 7
    B = wl.fill_values(rng, K * N, False).reshape(K, N)
    rowptr = np.arange(K + 1, dtype=np.int32)
    colidx = np.arange(K, dtype=np.int32)
    C, BND = oracle.spmm_csr(K, K, N, rowptr, colidx, np.ones(K, np.float32), B)
    assert np.array_equal(C.astype(np.float32), B)
    assert np.array_equal(BND, np.abs(B.astype(np.float64)))


def test_permutation_and_diagonal_scaling():
    # A = diag(d) * P : row i of C is d[i] * B[perm[i]]  (catches B[i] vs B[col])
    rng = np.random.default_rng(4)
    K, N = 23, 5
    B = wl.fill_values(rng, K * N, False).reshape(K, N)
    perm = rng.permutation(K).astype(np.int32)
    d = wl.fill_values(rng, K, False)
    C, _ = oracle.spmm_csr(K, K, N, np.arange(K + 1, dtype=np.int32), perm, d, B)
    assert np.array_equal(C, d.astype(np.float64)[:, None] * B[perm].astype(np.float64))


def test_ones_operand_gives_row_sums():
    rng = np.random.default_rng(5)
    M, K, N = 31, 40, 3
    rowptr, colidx, vals = random_csr(rng, M, K, 0.25, integer=True)
    C, _ = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, np.ones((K, N), np.float32))
    sums = np.array([vals[rowptr[i]:rowptr[i + 1]].astype(np.float64).sum() for i in range(M)])
    assert np.array_equal(C, np.repeat(sums[:, None], N, axis=1))


def test_linearity_in_A_exact_on_integers():
    rng = np.random.default_rng(6)
    M, K, N = 20, 30, 6
    rowptr, colidx, vals = random_csr(rng, M, K, 0.5, integer=True)
    B = wl.fill_values(rng, K * N, True).reshape(K, N)
    keep = rng.random(colidx.size) < 0.5
    v1 = np.where(keep, vals, 0).astype(np.float32)
    v2 = np.where(keep, 0, vals).astype(np.float32)
    C, _ = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, B)
    C1, _ = oracle.spmm_csr(M, K, N, rowptr, colidx, v1, B)
    C2, _ = oracle.spmm_csr(M, K, N, rowptr, colidx, v2, B)
    assert np.array_equal(C, C1 + C2)


def test_column_slices_of_B_give_column_slices_of_C():
    rng = np.random.default_rng(8)
    M, K, N = 25, 19, 12
    rowptr, colidx, vals = random_csr(rng, M, K, 0.3)
    B = wl.fill_values(rng, K * N, False).reshape(K, N)
    C, BND = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, B)
    Cs, BNDs = oracle.spmm_csr(M, K, 5, rowptr, colidx, vals, np.ascontiguousarray(B[:, 3:8]))
    assert np.array_equal(Cs, C[:, 3:8])
    assert np.array_equal(BNDs, BND[:, 3:8])


def test_row_permutation_of_A_permutes_C():
    rng = np.random.default_rng(9)
    M, K, N = 16, 21, 4
    rowptr, colidx, vals = random_csr(rng, M, K, 0.3)
    B = wl.fill_values(rng, K * N, False).reshape(K, N)
    C, _ = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, B)
    perm = rng.permutation(M)
    ln = np.diff(rowptr)[perm]
    rp2 = np.zeros(M + 1, np.int32)
    rp2[1:] = np.cumsum(ln)
    ci2 = np.concatenate([colidx[rowptr[i]:rowptr[i + 1]] for i in perm]).astype(np.int32)
    va2 = np.concatenate([vals[rowptr[i]:rowptr[i + 1]] for i in perm]).astype(np.float32)
    C2, _ = oracle.spmm_csr(M, K, N, rp2, ci2, va2, B)
    assert np.array_equal(C2, C[perm])


def test_unsorted_and_duplicate_columns_just_add():
    # row 0 holds column 2 twice and out of order; integer values => exact
    rowptr = np.array([0, 4, 5], dtype=np.int32)
    colidx = np.array([3, 2, 0, 2, 1], dtype=np.int32)
    vals = np.array([1, 2, -1, 2, 1], dtype=np.float32)
    B = np.arange(8, dtype=np.float32).reshape(4, 2)
    C, _ = oracle.spmm_csr(2, 4, 2, rowptr, colidx, vals, B)
    A = np.array([[-1, 0, 4, 1], [0, 1, 0, 0]], dtype=np.float64)
    assert np.array_equal(C, A @ B.astype(np.float64))


@pytest.mark.parametrize("name", ["uniform10", "uniform10_int", "powerlaw"])
def test_agrees_with_scipy_on_named_workloads(name):
    # independent library routine: scipy's csr @ dense in float64
    p = wl.make_problem(name, scale_down=8 if name == "powerlaw" else 1)
    C, BND = oracle.spmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B)
    A = sp.csr_matrix((p.vals.astype(np.float64), p.colidx, p.rowptr), shape=(p.M, p.K))
    ref = A @ p.B.astype(np.float64)
    absA = sp.csr_matrix((np.abs(p.vals.astype(np.float64)), p.colidx, p.rowptr), shape=(p.M, p.K))
    scale = absA @ np.abs(p.B.astype(np.float64))
    assert np.all(np.abs(C - ref) <= 1e-12 * scale)
    assert np.allclose(BND, scale, rtol=1e-12, atol=0)
    assert np.all(np.abs(C) <= BND)
    if name.endswith("_int"):
        assert np.array_equal(C, ref)


def test_bound_is_result_of_absolute_operands():
    rng = np.random.default_rng(11)
    M, K, N = 14, 18, 5
    rowptr, colidx, vals = random_csr(rng, M, K, 0.4)
    B = wl.fill_values(rng, K * N, False).reshape(K, N)
    _, BND = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, B)
    Cabs, _ = oracle.spmm_csr(M, K, N, rowptr, colidx, np.abs(vals), np.abs(B))
    assert np.array_equal(BND, Cabs)


def test_selected_rows_and_threads_agree_with_full_result():
    p = wl.make_problem("powerlaw", scale_down=16)
    C, BND = oracle.spmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B)
    C4, BND4 = oracle.spmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, nthreads=4)
    assert np.array_equal(C, C4) and np.array_equal(BND, BND4)
    rows = np.array([0, 5, p.M - 1, 77, 5], dtype=np.int64)
    Cr, BNDr = oracle.spmm_csr_rows(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, rows)
    assert np.array_equal(Cr, C[rows]) and np.array_equal(BNDr, BND[rows])


def test_rejects_malformed_input():
    B = np.zeros((3, 2), np.float32)
    with pytest.raises(ValueError):
        oracle.spmm_csr(2, 3, 2, np.array([0, 2, 1], np.int32), np.zeros(1, np.int32), np.zeros(1, np.float32), B)
    with pytest.raises(ValueError):
        oracle.spmm_csr(1, 3, 2, np.array([0, 1], np.int32), np.array([3], np.int32), np.ones(1, np.float32), B)
