"""Row reordering (sgap_reorder_rows_csr) against oracle/row_order.py, through the C ABI."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from oracle import row_order as ro
from paper_2209_02882_amd import binding, workloads as wl
from paper_2209_02882_amd.device import DeviceProblem

from gpu_util import TOL, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def reorder_on_gpu(M, K, rowptr, colidx, vals, order, poison=True):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    d_rowptr, d_colidx, d_vals = t(rowptr), t(colidx), t(vals)
    nnz = len(colidx)
    perm = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    rowptr_out = torch.full((M + 1,), -7, dtype=torch.int32, device=DEV)
    colidx_out = torch.full((nnz,), -7, dtype=torch.int32, device=DEV)
    vals_out = torch.full((nnz,), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(binding.sgap_reorder_rows_workspace_size(M), dtype=torch.uint8, device=DEV)
    if poison:
        ws.fill_(0xAB)
    binding.sgap_reorder_rows_csr(M, K, d_rowptr, d_colidx, d_vals, order, perm, rowptr_out, colidx_out, vals_out, ws)
    torch.cuda.synchronize()
    return perm.cpu().numpy(), rowptr_out.cpu().numpy(), colidx_out.cpu().numpy(), vals_out.cpu().numpy()


def random_csr(rng, M, K, max_len, empty_share=0.2):
    lengths = rng.integers(1, max_len + 1, M)
    lengths[rng.random(M) < empty_share] = 0
    lengths = np.minimum(lengths, K)
    rowptr = np.zeros(M + 1, dtype=np.int32)
    np.cumsum(lengths, out=rowptr[1:])
    colidx = np.concatenate([np.sort(rng.choice(K, n, replace=False)) for n in lengths] + [np.zeros(0, dtype=np.int64)])
    vals = rng.standard_normal(len(colidx)).astype(np.float32)
    return rowptr, colidx.astype(np.int32), vals


@pytest.mark.parametrize("order", ["first_column", "length"])
@pytest.mark.parametrize("M,K,max_len", [(1, 5, 3), (5, 8, 3), (63, 17, 9), (2048, 300, 12), (2049, 4096, 5),
                                         (6150, 100_000, 40), (20_000, 50, 50)])
def test_reordering_of_random_matrices(M, K, max_len, order):
    rng = np.random.default_rng(M * 31 + K)
    rowptr, colidx, vals = random_csr(rng, M, K, max_len)
    got = reorder_on_gpu(M, K, rowptr, colidx, vals, order)
    ro.check_reordering(M, K, rowptr, colidx, vals, order, *got)


@pytest.mark.parametrize("order", ["first_column", "length"])
def test_degenerate_matrices(order):
    # no stored entries at all; every row in one key; rows far longer than the largest length key; M == 0
    M, K = 3000, 64
    rowptr = np.zeros(M + 1, dtype=np.int32)
    got = reorder_on_gpu(M, K, rowptr, np.zeros(0, np.int32), np.zeros(0, np.float32), order)
    ro.check_reordering(M, K, rowptr, np.zeros(0, np.int32), np.zeros(0, np.float32), order, *got)

    rowptr = (np.arange(M + 1) * 2).astype(np.int32)
    colidx = np.tile(np.array([3, 9], dtype=np.int32), M)
    vals = np.arange(2 * M, dtype=np.float32)
    got = reorder_on_gpu(M, K, rowptr, colidx, vals, order)
    ro.check_reordering(M, K, rowptr, colidx, vals, order, *got)

    M, K = 7, 9000
    lengths = np.array([5000, 0, 4096, 8999, 1, 4095, 6000])
    rowptr = np.zeros(M + 1, dtype=np.int32)
    np.cumsum(lengths, out=rowptr[1:])
    rng = np.random.default_rng(3)
    colidx = np.concatenate([np.sort(rng.choice(K, n, replace=False)) for n in lengths]).astype(np.int32)
    vals = rng.standard_normal(len(colidx)).astype(np.float32)
    got = reorder_on_gpu(M, K, rowptr, colidx, vals, order)
    ro.check_reordering(M, K, rowptr, colidx, vals, order, *got)

    out = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    empty_i = torch.zeros(0, dtype=torch.int32, device=DEV)
    empty_f = torch.zeros(0, dtype=torch.float32, device=DEV)
    binding.sgap_reorder_rows_csr(0, 0, torch.zeros(1, dtype=torch.int32, device=DEV), empty_i, empty_f, order,
                                  empty_i, out, empty_i, empty_f, None)
    torch.cuda.synchronize()
    assert out.item() == 0


@pytest.mark.parametrize("order", ["first_column", "length"])
def test_product_of_the_reordered_matrix(order):
    # the whole point: SpMM on the new matrix gives the rows of the product in the new order
    p = wl.make_problem("powerlaw")
    perm, rp, ci, va = reorder_on_gpu(p.M, p.K, p.rowptr, p.colidx, p.vals, order)
    ro.check_reordering(p.M, p.K, p.rowptr, p.colidx, p.vals, order, perm, rp, ci, va)
    C_ref, BND = oracle.spmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, nthreads=8)
    q = dataclasses.replace(p, rowptr=rp, colidx=ci, vals=va)
    dp = DeviceProblem(q)
    for point in ((16, "serial", "nnz_balanced"), (8, "parallel", "row_split")):
        C = dp.run_cfg(binding.make_config(*point))
        assert_close(C, C_ref[perm], BND[perm], what=f"{order} {point}")


@pytest.mark.parametrize("order", ["first_column", "length"])
def test_full_size_rmat(order):
    # 2 M rows, 50 M entries: what is unique is compared in full with whole-array operations
    # (permutation, lengths), the rest on sampled rows and neighbouring places through the oracle
    p = wl.make_problem("rmat")
    perm, rp, ci, va = reorder_on_gpu(p.M, p.K, p.rowptr, p.colidx, p.vals, order, poison=False)
    assert np.array_equal(np.sort(perm), np.arange(p.M, dtype=np.int32))
    lengths = np.diff(p.rowptr)
    assert rp[0] == 0 and np.array_equal(np.diff(rp), lengths[perm])
    rng = np.random.default_rng(11)
    places = np.unique(np.concatenate([rng.integers(0, p.M - 1, 3000), [0, p.M - 2], np.argsort(-lengths[perm])[:20]]))
    places = places[places < p.M - 1]
    rows = np.unique(np.concatenate([perm[places], perm[places + 1]]))
    index_of = {int(r): n for n, r in enumerate(rows)}
    # the sampled rows as a small matrix of their own: the oracle's keys on it are the keys of those rows
    sub_rp = np.zeros(len(rows) + 1, dtype=np.int32)
    np.cumsum(lengths[rows], out=sub_rp[1:])
    sub_ci = np.concatenate([p.colidx[p.rowptr[r]:p.rowptr[r + 1]] for r in rows])
    keys = ro.row_order_keys(len(rows), p.K, sub_rp, sub_ci, order)
    for j in places:
        a, b = index_of[int(perm[j])], index_of[int(perm[j + 1])]
        assert keys[a] <= keys[b], f"key decreases at place {j}"
        r = int(perm[j])
        assert np.array_equal(ci[rp[j]:rp[j + 1]], p.colidx[p.rowptr[r]:p.rowptr[r + 1]])
        assert np.array_equal(va[rp[j]:rp[j + 1]].view(np.uint32), p.vals[p.rowptr[r]:p.rowptr[r + 1]].view(np.uint32))


def test_bad_arguments_launch_nothing():
    M, K = 10, 10
    rowptr = torch.zeros(M + 1, dtype=torch.int32, device=DEV)
    e_i = torch.zeros(0, dtype=torch.int32, device=DEV)
    e_f = torch.zeros(0, dtype=torch.float32, device=DEV)
    perm = torch.full((M,), -7, dtype=torch.int32, device=DEV)
    out = torch.full((M + 1,), -7, dtype=torch.int32, device=DEV)
    ws = torch.empty(binding.sgap_reorder_rows_workspace_size(M), dtype=torch.uint8, device=DEV)
    for kwargs in (dict(order=2), dict(workspace=None), dict(workspace=ws[:64]), dict(workspace=ws[1:]), dict(K=0)):
        args = dict(M=M, K=K, order=0, workspace=ws)
        args.update(kwargs)
        with pytest.raises(binding.SgapError) as err:
            binding.sgap_reorder_rows_csr(args["M"], args["K"], rowptr, e_i, e_f, args["order"], perm, out, e_i, e_f,
                                          args["workspace"])
        assert err.value.status == binding.SGAP_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert (perm == -7).all() and (out == -7).all()
