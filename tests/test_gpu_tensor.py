"""GPU parity of MTTKRP and TTM on compressed sparse fibers against the fp64
oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_02882_amd import binding
from paper_2209_02882_amd import workloads as wl
from paper_2209_02882_amd.device import POINTS, DeviceTensor3

from gpu_util import TOL, assert_close

pytestmark = pytest.mark.gpu

# (group size, strategy, schedule): slices or stored entries as the unit of work
MTTKRP_POINTS = [(g, st, sc) for sc in ("row_split", "nnz_balanced") for st in ("parallel", "serial")
                 for g in binding.GROUP_SIZES]


def mttkrp_reference(p, nthreads=8):
    return oracle.mttkrp_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, p.X1, p.X2,
                             nthreads=nthreads)


def tensor_from(I, K, L, J, fiber_counts, entry_counts, seed, integer=False):
    """A tensor with the given fibers per slice and entries per fiber, indices uniform distinct."""
    rng = np.random.default_rng(seed)
    fptr, fidx = wl.csr_from_lengths(rng, np.asarray(fiber_counts, dtype=np.int64), K)
    entry_counts = np.resize(np.asarray(entry_counts, dtype=np.int64), int(fptr[-1]))
    eptr, eidx = wl.csr_from_lengths(rng, entry_counts, L)
    vals = wl.fill_values(rng, int(eptr[-1]), integer)
    X1 = wl.fill_values(rng, K * J, integer).reshape(K, J)
    X2 = wl.fill_values(rng, L * J, integer).reshape(L, J)
    return wl.Tensor3Problem("custom", I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2)


@pytest.mark.parametrize("name,J", [("tensor3_small", None), ("tensor3_small_int", None), ("tensor3_small", 20),
                                    ("tensor3_small", 5), ("tensor3_small", 6), ("tensor3_small", 1),
                                    ("tensor3_small", 4), ("tensor3_small_int", 130), ("tensor3_small", 256),
                                    ("tensor3_small", 300)])
def test_mttkrp_every_point_matches_the_oracle(name, J):
    p = wl.make_tensor3(name, J=J)
    ref, bnd = mttkrp_reference(p)
    dt = DeviceTensor3(p)
    for g, st, sc in MTTKRP_POINTS:
        print("  mttkrp", name, J, g, st, sc, flush=True)
        assert_close(dt.run_mttkrp(g, st, sc), ref, bnd, exact=name.endswith("_int"),
                     what=f"{name} J={J} g={g} {st} {sc}")


@pytest.mark.parametrize("case", ["one_slice", "long_fibers", "many_fibers", "ragged_tail", "all_empty",
                                  "single_entries", "runs_without_entries", "several_tiles"])
def test_mttkrp_shapes_at_the_edges(case):
    if case == "one_slice":
        p = tensor_from(1, 40, 50, 32, [7], [1, 3, 9, 2, 33, 1, 4], 1)
    elif case == "long_fibers":  # fibers longer than any run of chunk lanes, by a ragged amount
        p = tensor_from(37, 64, 400, 32, [3] * 37, [70, 1, 129, 64, 65, 8, 9], 2, integer=True)
    elif case == "many_fibers":  # one slice with far more fibers than lanes, the rest empty or short
        p = tensor_from(20, 600, 90, 24, [0, 517] + [0, 2] * 9, [2, 5, 1], 3)
    elif case == "ragged_tail":  # slice counts that leave the last workgroup and the last group partly filled
        p = tensor_from(259, 80, 80, 12, [1, 0, 4, 2, 9, 0, 3] * 37, [1, 2, 3, 4, 5], 4, integer=True)
    elif case == "all_empty":
        p = tensor_from(300, 10, 10, 16, [0] * 300, [1], 5)
    elif case == "runs_without_entries":
        # more slices without fibers and more fibers without entries in a row than a pointer window of the
        # nnz-balanced kernel holds (1,025), at the start, in the middle and at the end
        fibers = [0] * 1500 + [3] + [0] * 2100 + [1400, 2] + [0] * 1100 + [5] + [0] * 1030
        entries = [0] * 2 + [4] + [0] * 1200 + [1, 2, 9] + [0] * 190 + [3, 0, 0, 1]
        p = tensor_from(len(fibers), 2000, 70, 32, fibers, entries, 7, integer=True)
    elif case == "several_tiles":
        # 5,000 and some entries: five tiles of the nnz-balanced kernel, the last one ragged; slices and fibers
        # that straddle tile ends
        p = tensor_from(91, 300, 500, 40, [1, 0, 7, 2, 19, 0, 3] * 13, [30, 1, 2, 90, 5, 41, 8, 3], 8, integer=True)
    else:
        p = tensor_from(1000, 50, 60, 8, [1] * 1000, [1], 6, integer=True)
    ref, bnd = mttkrp_reference(p)
    dt = DeviceTensor3(p)
    exact = case in ("long_fibers", "ragged_tail", "single_entries", "runs_without_entries", "several_tiles")
    for g, st, sc in MTTKRP_POINTS:
        print("  mttkrp", case, g, st, sc, flush=True)
        assert_close(dt.run_mttkrp(g, st, sc), ref, bnd, exact=exact, what=f"{case} g={g} {st} {sc}")


@pytest.mark.parametrize("seed", range(16))
def test_mttkrp_random_shapes(seed):
    # seeded random tensors: slices without fibers, fibers without entries, a heavy slice now and then,
    # any number of columns; three random points per schedule
    rng = np.random.default_rng(1000 + seed)
    I = int(rng.integers(1, 3000))
    K = int(rng.integers(1, 400))
    L = int(rng.integers(1, 400))
    J = int(rng.choice([1, 3, 4, 8, 12, 32, 33, 64, 100, 256]))
    fibers = rng.geometric(1.0 / float(rng.uniform(1.0, 6.0)), size=I) - 1
    if seed % 3 == 0:
        fibers[rng.integers(0, I)] = K
    fibers = np.minimum(fibers, K)
    fibers[rng.random(I) < rng.uniform(0.0, 0.7)] = 0
    entries = np.minimum(rng.geometric(1.0 / float(rng.uniform(1.0, 20.0)), size=int(fibers.sum()) + 1) - (seed % 2), L)
    entries = np.maximum(entries, 0)
    p = tensor_from(I, K, L, J, fibers, entries, 2000 + seed, integer=True)
    ref, bnd = mttkrp_reference(p)
    dt = DeviceTensor3(p)
    for sc in ("row_split", "nnz_balanced"):
        for _ in range(3):
            g = int(rng.choice(binding.GROUP_SIZES))
            st = str(rng.choice(["parallel", "serial"]))
            print("  mttkrp random", seed, I, K, L, J, p.fibers, p.nnz, g, st, sc, flush=True)
            assert_close(dt.run_mttkrp(g, st, sc), ref, bnd, exact=True, what=f"seed {seed} g={g} {st} {sc}")


def test_mttkrp_unsorted_and_repeated_indices_just_add():
    p = wl.make_tensor3("tensor3_small_int")
    rng = np.random.default_rng(9)
    # shuffle the entries inside every fiber and repeat some third indices
    eidx = p.eidx.copy()
    vals = p.vals.copy()
    for f in range(p.fibers):
        a, b = p.eptr[f], p.eptr[f + 1]
        perm = rng.permutation(b - a)
        eidx[a:b] = eidx[a:b][perm]
        vals[a:b] = vals[a:b][perm]
        if b - a > 2:
            eidx[a + 1] = eidx[a]
    p.eidx, p.vals = eidx, vals
    # repeated second indices inside a slice as well
    fidx = p.fidx.copy()
    for i in range(p.I):
        if p.fptr[i + 1] - p.fptr[i] > 1:
            fidx[p.fptr[i] + 1] = fidx[p.fptr[i]]
    p.fidx = fidx
    ref, bnd = mttkrp_reference(p)
    dt = DeviceTensor3(p)
    for g, st, sc in MTTKRP_POINTS:
        assert_close(dt.run_mttkrp(g, st, sc), ref, bnd, exact=True, what=f"unsorted g={g} {st} {sc}")


def test_mttkrp_unaligned_operands_take_narrower_loads():
    p = wl.make_tensor3("tensor3_small")
    ref, bnd = mttkrp_reference(p)
    dt = DeviceTensor3(p)
    # an operand that starts 4 bytes past a 16-byte boundary
    pad = torch.empty(p.L * p.J + 1, dtype=torch.float32, device="cuda:0")
    dt.X2 = pad[1:].view(p.L, p.J)
    dt.X2.copy_(torch.from_numpy(p.X2))
    assert dt.X2.data_ptr() % 16 == 4
    for g, st, sc in [(1, "parallel", "row_split"), (8, "parallel", "row_split"), (4, "serial", "row_split"),
                      (8, "parallel", "nnz_balanced"), (16, "serial", "nnz_balanced")]:
        assert_close(dt.run_mttkrp(g, st, sc), ref, bnd, what=f"unaligned g={g} {st} {sc}")


def test_mttkrp_full_size():
    p = wl.make_tensor3("tensor3")
    print(p.stats(), flush=True)
    ref, bnd = mttkrp_reference(p, nthreads=16)
    dt = DeviceTensor3(p)
    for g, st, sc in MTTKRP_POINTS:
        print("  mttkrp full size", g, st, sc, flush=True)
        assert_close(dt.run_mttkrp(g, st, sc), ref, bnd, what=f"tensor3 g={g} {st} {sc}")


def test_mttkrp_rejects_bad_arguments():
    p = wl.make_tensor3("tensor3_small")
    dt = DeviceTensor3(p)
    Y = torch.empty((p.I, p.J), dtype=torch.float32, device="cuda:0")
    with pytest.raises(binding.SgapError):
        dt.launch_mttkrp(Y, 3, "parallel")
    with pytest.raises(binding.SgapError):
        binding.sgap_mttkrp_csf(p.I, p.K, p.L, p.J, dt.fptr, dt.fidx, dt.eptr, dt.eidx, dt.vals, dt.X1, dt.X2, Y,
                                4, 7)
    with pytest.raises(binding.SgapError):
        binding.sgap_mttkrp_csf_ex(p.I, p.K, p.L, p.J, dt.fptr, dt.fidx, dt.eptr, dt.eidx, dt.vals, dt.X1, dt.X2, Y,
                                   4, binding.SGAP_REDUCE_SERIAL, 2)


@pytest.mark.parametrize("name", ["tensor3_small", "tensor3_small_int"])
def test_ttm_every_point_matches_the_oracle(name):
    p = wl.make_tensor3(name)
    ref, bnd = oracle.ttm_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, p.X2, nthreads=8)
    dt = DeviceTensor3(p)
    for g, st, sc in POINTS:
        assert_close(dt.run_ttm(g, st, sc), ref, bnd, exact=name.endswith("_int"), what=f"ttm {name} g={g} {st} {sc}")


def test_ttm_full_size():
    p = wl.make_tensor3("tensor3")
    ref, bnd = oracle.ttm_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, p.X2, nthreads=16)
    dt = DeviceTensor3(p)
    for g, st, sc in [(8, "parallel", "row_split"), (16, "serial", "nnz_balanced"), (8, "parallel", "nnz_balanced"),
                      (2, "serial", "row_split")]:
        print("  ttm full size", g, st, sc, flush=True)
        assert_close(dt.run_ttm(g, st, sc), ref, bnd, what=f"ttm tensor3 g={g} {st} {sc}")


def test_mttkrp_wide_factor_offsets_need_64_bits():
    # L*J*4 >= 2^32: offsets into X2 do not fit 32 bits, the fast address path must not be taken
    I, K, L, J = 200, 50, 1 << 22, 256
    rng = np.random.default_rng(31)
    p = tensor_from(I, K, L, J, rng.integers(0, 5, size=I), [1, 2, 7, 3], 31, integer=True)
    p.eidx[-1] = L - 1  # the far end of X2 is touched
    rows_used = np.unique(p.eidx)
    X2small = wl.fill_values(rng, rows_used.size * J, True).reshape(-1, J)
    X2 = torch.zeros((L, J), dtype=torch.float32, device="cuda:0")
    X2[torch.from_numpy(rows_used.astype(np.int64)).cuda()] = torch.from_numpy(X2small).cuda()
    # oracle on a compacted copy (same rows of X2, renumbered third indices)
    remap = np.searchsorted(rows_used, p.eidx).astype(np.int32)
    ref, bnd = oracle.mttkrp_csf(I, K, rows_used.size, J, p.fptr, p.fidx, p.eptr, remap, p.vals, p.X1, X2small)
    dev = {n: torch.from_numpy(getattr(p, n)).cuda() for n in ("fptr", "fidx", "eptr", "eidx", "vals", "X1")}
    for g, st in [(1, "parallel"), (8, "parallel"), (64, "parallel"), (4, "serial")]:
        Y = torch.full((I, J), float("nan"), device="cuda:0")
        binding.sgap_mttkrp_csf(I, K, L, J, dev["fptr"], dev["fidx"], dev["eptr"], dev["eidx"], dev["vals"], dev["X1"],
                                X2, Y, g, binding.STRATEGIES[st])
        torch.cuda.synchronize()
        assert_close(Y, ref, bnd, exact=True, what=f"64-bit offsets g={g} {st}")
