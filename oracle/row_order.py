"""CPU oracle of the row-reordering pass (test infrastructure, not part of the product).

The pass groups the rows of a CSR matrix by a coarse key (smaller key first, any order
inside a key) and writes the permuted copy; the paper's schedules (its Section 6) take
rows in stored order, and its Section 2.2 names the locality work a better order stands
for.  Several permutations are correct, so the oracle does not produce "the" answer: it
states the keys (plain integer arithmetic, one row at a time) and checks a claimed result:
  row_order_keys     the key of every row, as the interface defines it
  permute_rows_csr   the CSR copy that a given permutation implies (row by row)
  check_reordering   perm is a permutation, keys do not decrease along it, and the
                     three output arrays are exactly what permute_rows_csr gives
Pins (tests/test_oracle_reorder.py): a hand-worked example, the identity and reversal
permutations, and the SpMM oracle: the product of the permuted matrix equals the permuted
rows of the product.
"""
from __future__ import annotations

import numpy as np

BUCKETS = 4097  # keys 0 .. 4096


def row_order_keys(M, K, rowptr, colidx, order: str) -> np.ndarray:
    """order = "first_column": floor(first stored column * 4096 / K); "length": 4096 - min(entries, 4096);
    a row without stored entries has key 4096 either way."""
    keys = np.empty(M, dtype=np.int64)
    for i in range(M):
        p0, p1 = int(rowptr[i]), int(rowptr[i + 1])
        if p1 <= p0:
            keys[i] = BUCKETS - 1
        elif order == "first_column":
            keys[i] = int(colidx[p0]) * (BUCKETS - 1) // K
        elif order == "length":
            keys[i] = (BUCKETS - 1) - min(p1 - p0, BUCKETS - 1)
        else:
            raise ValueError("unknown order")
    return keys


def permute_rows_csr(rowptr, colidx, vals, perm):
    """Row j of the result is row perm[j] of the input, entries in their stored order."""
    M = len(perm)
    rp = np.zeros(M + 1, dtype=np.int32)
    ci, va = [], []
    for j in range(M):
        i = int(perm[j])
        p0, p1 = int(rowptr[i]), int(rowptr[i + 1])
        ci.extend(colidx[p0:p1].tolist())
        va.extend(vals[p0:p1].tolist())
        rp[j + 1] = rp[j] + (p1 - p0)
    return rp, np.asarray(ci, dtype=np.int32), np.asarray(va, dtype=np.float32)


def check_reordering(M, K, rowptr, colidx, vals, order, perm, rowptr_out, colidx_out, vals_out) -> None:
    """Raises AssertionError naming what is wrong with a claimed result."""
    perm = np.asarray(perm)
    assert perm.shape == (M,), "perm must have M entries"
    seen = np.zeros(M, dtype=bool)
    for j in range(M):
        i = int(perm[j])
        assert 0 <= i < M and not seen[i], f"perm[{j}] = {i} is out of range or repeated"
        seen[i] = True
    keys = row_order_keys(M, K, rowptr, colidx, order)
    along = keys[perm] if M else keys
    for j in range(1, M):
        assert along[j - 1] <= along[j], f"key decreases at place {j}: {along[j - 1]} then {along[j]}"
    rp, ci, va = permute_rows_csr(rowptr, colidx, vals, perm)
    assert np.array_equal(np.asarray(rowptr_out), rp), "rowptr_out differs"
    assert np.array_equal(np.asarray(colidx_out), ci), "colidx_out differs"
    assert np.array_equal(np.asarray(vals_out).view(np.uint32), va.view(np.uint32)), "vals_out differs"
