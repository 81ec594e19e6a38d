"""Pins of the row-reordering oracle (oracle/row_order.py): no GPU."""
import numpy as np
import pytest

import oracle
from oracle import row_order as ro


def small_matrix():
    # 5 x 8, rows: [2, 7], [], [0], [5, 6, 7], [4]
    rowptr = np.array([0, 2, 2, 3, 6, 7], dtype=np.int32)
    colidx = np.array([2, 7, 0, 5, 6, 7, 4], dtype=np.int32)
    vals = np.array([1.0, 2.0, 3.0, 4.0, 5.0, 6.0, 7.0], dtype=np.float32)
    return 5, 8, rowptr, colidx, vals


def test_keys_by_hand():
    M, K, rowptr, colidx, vals = small_matrix()
    # first columns 2, -, 0, 5, 4 of K = 8: floor(c * 4096 / 8) = 512 c; the row without entries gets 4096
    assert ro.row_order_keys(M, K, rowptr, colidx, "first_column").tolist() == [1024, 4096, 0, 2560, 2048]
    # lengths 2, 0, 1, 3, 1: 4096 - length; the row without entries gets 4096
    assert ro.row_order_keys(M, K, rowptr, colidx, "length").tolist() == [4094, 4096, 4095, 4093, 4095]
    # a row of 5,000 entries shares key 0 with every row of at least 4,096
    rp = np.array([0, 5000, 9096], dtype=np.int32)
    ci = np.concatenate([np.arange(5000), np.arange(4096)]).astype(np.int32)
    assert ro.row_order_keys(2, 6000, rp, ci, "length").tolist() == [0, 0]
    with pytest.raises(ValueError):
        ro.row_order_keys(M, K, rowptr, colidx, "other")


def test_permuted_copy_by_hand():
    M, K, rowptr, colidx, vals = small_matrix()
    rp, ci, va = ro.permute_rows_csr(rowptr, colidx, vals, [3, 0, 4, 2, 1])
    assert rp.tolist() == [0, 3, 5, 6, 7, 7]
    assert ci.tolist() == [5, 6, 7, 2, 7, 4, 0]
    assert va.tolist() == [4.0, 5.0, 6.0, 1.0, 2.0, 7.0, 3.0]
    # the identity gives the matrix back
    rp, ci, va = ro.permute_rows_csr(rowptr, colidx, vals, np.arange(M))
    assert np.array_equal(rp, rowptr) and np.array_equal(ci, colidx) and np.array_equal(va, vals)


def test_checker_accepts_every_valid_order_and_names_each_mistake():
    M, K, rowptr, colidx, vals = small_matrix()
    for order, perms in (("first_column", ([2, 0, 4, 3, 1],)), ("length", ([3, 0, 2, 4, 1], [3, 0, 4, 2, 1]))):
        for perm in perms:
            out = ro.permute_rows_csr(rowptr, colidx, vals, perm)
            ro.check_reordering(M, K, rowptr, colidx, vals, order, perm, *out)
    perm = [3, 0, 2, 4, 1]
    rp, ci, va = ro.permute_rows_csr(rowptr, colidx, vals, perm)
    with pytest.raises(AssertionError, match="repeated"):
        ro.check_reordering(M, K, rowptr, colidx, vals, "length", [3, 0, 2, 2, 1], rp, ci, va)
    with pytest.raises(AssertionError, match="key decreases"):
        bad = [0, 3, 2, 4, 1]
        ro.check_reordering(M, K, rowptr, colidx, vals, "length", bad, *ro.permute_rows_csr(rowptr, colidx, vals, bad))
    with pytest.raises(AssertionError, match="rowptr_out"):
        ro.check_reordering(M, K, rowptr, colidx, vals, "length", perm, rp + 1, ci, va)
    with pytest.raises(AssertionError, match="colidx_out"):
        ro.check_reordering(M, K, rowptr, colidx, vals, "length", perm, rp, ci[::-1].copy(), va)
    with pytest.raises(AssertionError, match="vals_out"):
        ro.check_reordering(M, K, rowptr, colidx, vals, "length", perm, rp, ci, -va)


def test_product_of_the_permuted_matrix_is_the_permuted_product():
    rng = np.random.default_rng(7)
    M, K, N = 40, 23, 6
    lengths = rng.integers(0, 9, M)
    rowptr = np.zeros(M + 1, dtype=np.int32)
    np.cumsum(lengths, out=rowptr[1:])
    colidx = np.concatenate([np.sort(rng.choice(K, n, replace=False)) for n in lengths]).astype(np.int32)
    vals = rng.integers(-2, 3, len(colidx)).astype(np.float32)
    B = rng.integers(-2, 3, (K, N)).astype(np.float32)
    C, _ = oracle.spmm_csr(M, K, N, rowptr, colidx, vals, B)
    for order in ("first_column", "length"):
        keys = ro.row_order_keys(M, K, rowptr, colidx, order)
        perm = np.argsort(keys, kind="stable")
        rp, ci, va = ro.permute_rows_csr(rowptr, colidx, vals, perm)
        ro.check_reordering(M, K, rowptr, colidx, vals, order, perm, rp, ci, va)
        Cp, _ = oracle.spmm_csr(M, K, N, rp, ci, va, B)
        assert np.array_equal(Cp, C[perm])
