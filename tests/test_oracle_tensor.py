"""Pins of the MTTKRP and TTM oracles (CPU only): a hand-worked example, the
definitions as numpy einsum over the densified tensor and as a loop over
coordinate triples, exact integer inputs, special cases that reduce to SpMM
or to a plain product, linearity, and permutation of the slices."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2209_02882_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_csf(rng, I, K, L, fiber_density, entry_density, integer=False):
    """Small random tensor drawn through a dense mask (not through the workload generator)."""
    mask = rng.random((I, K, L)) < entry_density
    mask &= (rng.random((I, K)) < fiber_density)[:, :, None]
    if I > 2:
        mask[rng.integers(0, I)] = False  # an empty slice
    fibers = mask.any(axis=2)
    fptr = np.zeros(I + 1, dtype=np.int32)
    fptr[1:] = np.cumsum(fibers.sum(1))
    ii, kk = np.nonzero(fibers)
    fidx = kk.astype(np.int32)
    eptr = np.zeros(fidx.size + 1, dtype=np.int32)
    eptr[1:] = np.cumsum(mask[ii, kk].sum(1))
    eidx = np.nonzero(mask[ii, kk])[1].astype(np.int32)
    vals = wl.fill_values(rng, eidx.size, integer)
    return fptr, fidx, eptr, eidx, vals


def coordinates(fptr, fidx, eptr, eidx):
    """(i, k, l) of every stored entry, in storage order."""
    fiber_slice = np.repeat(np.arange(fptr.size - 1), np.diff(fptr))
    entry_fiber = np.repeat(np.arange(fidx.size), np.diff(eptr))
    return fiber_slice[entry_fiber], fidx[entry_fiber], eidx, entry_fiber


def densify(I, K, L, fptr, fidx, eptr, eidx, vals):
    A = np.zeros((I, K, L), dtype=np.float64)
    i, k, l, _ = coordinates(fptr, fidx, eptr, eidx)
    np.add.at(A, (i, k, l), vals.astype(np.float64))
    return A


def read_golden():
    d = {}
    with open(os.path.join(GOLDEN, "tensor_2x2x3_by_hand.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            d[k] = v
    return d


def test_golden_hand_worked_example():
    d = read_golden()
    I, K, L, J = (int(d[n][0]) for n in "IKLJ")
    csf = [np.array(d[n], dtype=np.int32) for n in ("fptr", "fidx", "eptr", "eidx")]
    vals = np.array(d["vals"], dtype=np.float32)
    X1 = np.array(d["X1"], dtype=np.float32).reshape(K, J)
    X2 = np.array(d["X2"], dtype=np.float32).reshape(L, J)
    Y, BND = oracle.mttkrp_csf(I, K, L, J, *csf, vals, X1, X2)
    assert np.array_equal(Y.ravel(), np.array(d["mttkrp"], dtype=np.float64))
    assert np.array_equal(BND.ravel(), np.array(d["mttkrp_BND"], dtype=np.float64))
    Yf, BNDf = oracle.ttm_csf(I, K, L, J, *csf, vals, X2)
    assert np.array_equal(Yf.ravel(), np.array(d["ttm"], dtype=np.float64))
    assert np.array_equal(BNDf.ravel(), np.array(d["ttm_BND"], dtype=np.float64))


@pytest.mark.parametrize("seed,shape", [(1, (5, 4, 6, 3)), (2, (9, 7, 5, 8)), (3, (1, 1, 1, 1)), (4, (6, 3, 17, 5))])
def test_mttkrp_is_the_einsum_of_the_dense_tensor(seed, shape):
    I, K, L, J = shape
    rng = np.random.default_rng(seed)
    csf = random_csf(rng, I, K, L, 0.7, 0.5)
    X1 = wl.fill_values(rng, K * J, False).reshape(K, J)
    X2 = wl.fill_values(rng, L * J, False).reshape(L, J)
    Y, BND = oracle.mttkrp_csf(I, K, L, J, *csf, X1, X2)
    A = densify(I, K, L, *csf)
    ref = np.einsum("ikl,kj,lj->ij", A, X1.astype(np.float64), X2.astype(np.float64))
    assert np.allclose(Y, ref, rtol=0, atol=1e-12)
    refb = np.einsum("ikl,kj,lj->ij", np.abs(A), np.abs(X1).astype(np.float64), np.abs(X2).astype(np.float64))
    assert np.allclose(BND, refb, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed,shape", [(1, (5, 4, 6, 3)), (2, (9, 7, 5, 8)), (3, (1, 1, 1, 1)), (4, (6, 3, 17, 5))])
def test_ttm_is_the_einsum_of_the_dense_tensor(seed, shape):
    I, Jd, K, L = shape
    rng = np.random.default_rng(seed)
    csf = random_csf(rng, I, Jd, K, 0.7, 0.5)
    D = wl.fill_values(rng, K * L, False).reshape(K, L)
    Yf, BND = oracle.ttm_csf(I, Jd, K, L, *csf, D)
    A = densify(I, Jd, K, *csf)
    ref = np.einsum("ijk,kl->ijl", A, D.astype(np.float64))
    fiber_slice = np.repeat(np.arange(I), np.diff(csf[0]))
    assert np.allclose(Yf, ref[fiber_slice, csf[1]], rtol=0, atol=1e-12)
    # rows of Y without a stored fiber are zero, so nothing is lost by keeping the stored ones
    stored = np.zeros((I, Jd), dtype=bool)
    stored[fiber_slice, csf[1]] = True
    assert not ref[~stored].any()
    refb = np.einsum("ijk,kl->ijl", np.abs(A), np.abs(D).astype(np.float64))
    assert np.allclose(BND, refb[fiber_slice, csf[1]], rtol=0, atol=1e-12)


def test_mttkrp_triple_loop_over_coordinates_exact_on_integers():
    rng = np.random.default_rng(7)
    I, K, L, J = 7, 5, 6, 4
    csf = random_csf(rng, I, K, L, 0.8, 0.6, integer=True)
    X1 = wl.fill_values(rng, K * J, True).reshape(K, J)
    X2 = wl.fill_values(rng, L * J, True).reshape(L, J)
    Y, _ = oracle.mttkrp_csf(I, K, L, J, *csf, X1, X2)
    ref = [[0] * J for _ in range(I)]
    i, k, l, _ = coordinates(*csf[:4])
    for e in range(i.size):
        for j in range(J):
            ref[i[e]][j] += int(csf[4][e]) * int(X1[k[e], j]) * int(X2[l[e], j])
    assert np.array_equal(Y, np.array(ref, dtype=np.float64))


def test_all_ones_factors_turn_mttkrp_into_row_sums():
    # X1 = X2 = 1: Y[i, j] = sum of the slice's values, for every j
    p = wl.make_tensor3("tensor3_small_int")
    ones1, ones2 = np.ones((p.K, p.J), np.float32), np.ones((p.L, p.J), np.float32)
    Y, _ = oracle.mttkrp_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, ones1, ones2)
    fiber_sums = np.add.reduceat(np.concatenate([p.vals.astype(np.float64), [0.0]]), p.eptr[:-1])
    fiber_sums[np.diff(p.eptr) == 0] = 0.0
    slice_sums = np.zeros(p.I)
    np.add.at(slice_sums, np.repeat(np.arange(p.I), np.diff(p.fptr)), fiber_sums)
    assert np.array_equal(Y, np.repeat(slice_sums[:, None], p.J, axis=1))


def test_x1_all_ones_turns_mttkrp_into_spmm_of_the_flattened_tensor():
    # with X1 = 1 the second index drops out: Y = A_(i, l) * X2 where A_(i,l) sums over k
    p = wl.make_tensor3("tensor3_small")
    ones1 = np.ones((p.K, p.J), np.float32)
    Y, _ = oracle.mttkrp_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, ones1, p.X2)
    i, _, l, _ = coordinates(p.fptr, p.fidx, p.eptr, p.eidx)
    flat = sp.coo_matrix((p.vals.astype(np.float64), (i, l)), shape=(p.I, p.L)).tocsr()
    ref = flat @ p.X2.astype(np.float64)
    assert np.allclose(Y, ref, rtol=0, atol=1e-11)


def test_one_entry_per_fiber_mttkrp_is_a_product_of_three_numbers():
    rng = np.random.default_rng(11)
    I, K, L, J = 6, 4, 5, 3
    fptr = np.arange(I + 1, dtype=np.int32)          # one fiber per slice
    fidx = rng.integers(0, K, I).astype(np.int32)
    eptr = np.arange(I + 1, dtype=np.int32)          # one entry per fiber
    eidx = rng.integers(0, L, I).astype(np.int32)
    vals = wl.fill_values(rng, I, False)
    X1 = wl.fill_values(rng, K * J, False).reshape(K, J)
    X2 = wl.fill_values(rng, L * J, False).reshape(L, J)
    Y, BND = oracle.mttkrp_csf(I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2)
    ref = vals.astype(np.float64)[:, None] * X1[fidx].astype(np.float64) * X2[eidx].astype(np.float64)
    assert np.array_equal(Y, ref)
    assert np.array_equal(BND, np.abs(ref))


def test_ttm_equals_the_spmm_oracle_and_scipy_on_the_fiber_level():
    p = wl.make_tensor3("tensor3_small")
    Yf, BND = oracle.ttm_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, p.X2)
    A = sp.csr_matrix((p.vals.astype(np.float64), p.eidx, p.eptr), shape=(p.fibers, p.L))
    assert np.allclose(Yf, A @ p.X2.astype(np.float64), rtol=0, atol=1e-12)
    C, B2 = oracle.spmm_csr(p.fibers, p.L, p.J, p.eptr, p.eidx, p.vals, p.X2)
    assert np.array_equal(Yf, C) and np.array_equal(BND, B2)


def test_linearity_in_the_values_and_permutation_of_slices():
    p = wl.make_tensor3("tensor3_small_int")
    args = (p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx)
    Y, _ = oracle.mttkrp_csf(*args, p.vals, p.X1, p.X2)
    Y3, _ = oracle.mttkrp_csf(*args, 3 * p.vals, p.X1, p.X2)
    assert np.array_equal(Y3, 3 * Y)
    # reverse the order of the slices: rows of Y reverse
    fl = np.diff(p.fptr)[::-1]
    fptr_r = np.zeros(p.I + 1, dtype=np.int32)
    fptr_r[1:] = np.cumsum(fl)
    order = np.concatenate([np.arange(p.fptr[i], p.fptr[i + 1]) for i in range(p.I - 1, -1, -1)]).astype(np.int64)
    el = np.diff(p.eptr)[order]
    eptr_r = np.zeros(order.size + 1, dtype=np.int32)
    eptr_r[1:] = np.cumsum(el)
    ent = np.concatenate([np.arange(p.eptr[f], p.eptr[f + 1]) for f in order]).astype(np.int64)
    Yr, _ = oracle.mttkrp_csf(p.I, p.K, p.L, p.J, fptr_r, p.fidx[order], eptr_r, p.eidx[ent], p.vals[ent], p.X1, p.X2)
    assert np.array_equal(Yr, Y[::-1])


def test_empty_tensor_and_empty_slices_give_zero_rows():
    I, K, L, J = 4, 3, 3, 5
    z = np.zeros(I + 1, dtype=np.int32)
    e = np.zeros(0, dtype=np.int32)
    X1 = np.ones((K, J), np.float32)
    X2 = np.ones((L, J), np.float32)
    Y, BND = oracle.mttkrp_csf(I, K, L, J, z, e, np.zeros(1, np.int32), e, np.zeros(0, np.float32), X1, X2)
    assert not Y.any() and not BND.any()


def test_generator_invariants():
    p = wl.make_tensor3("tensor3_small")
    assert p.fptr[0] == 0 and p.eptr[0] == 0 and p.fptr[-1] == p.fidx.size and p.eptr[-1] == p.eidx.size
    assert (np.diff(p.eptr) >= 1).all(), "no empty fibers"
    assert (np.diff(p.fptr) == 0).any(), "some empty slices"
    for i in range(p.I):
        k = p.fidx[p.fptr[i]:p.fptr[i + 1]]
        assert (np.diff(k) > 0).all()
    for f in range(0, p.fibers, 37):
        l = p.eidx[p.eptr[f]:p.eptr[f + 1]]
        assert (np.diff(l) > 0).all()
    q = wl.make_tensor3("tensor3_small")
    assert np.array_equal(p.eidx, q.eidx) and np.array_equal(p.vals, q.vals) and np.array_equal(p.X1, q.X1)
