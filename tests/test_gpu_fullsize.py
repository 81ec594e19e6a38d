"""Full-size workloads in the launch configuration the benchmark times: the
whole result of the benchmark's best configuration and of one point of every
other kernel family against the oracle, element by element; all 28 points on
sampled output rows the oracle computes one by one, plus properties that hold
at any size (no element left unwritten)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_02882_amd import binding
from paper_2209_02882_amd import workloads as wl

from gpu_util import POINTS, TOL, DeviceProblem, sample_rows

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["stencil27", "rmat", "skewed"])
def test_full_size_sampled_rows(name):
    p = wl.make_problem(name)
    print(name, p.row_stats(), flush=True)
    dp = DeviceProblem(p)
    rows = sample_rows(p)
    C_ref, BND = oracle.spmm_csr_rows(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, rows)
    rows_t = torch.from_numpy(rows).cuda()
    C = torch.empty((p.M, p.N), dtype=torch.float32, device="cuda:0")
    for point in POINTS:
        print("  point", point, flush=True)
        dp.run(*point, C=C)
        assert not torch.isnan(C).any(), f"{name} {point}: element never written"
        got = C.index_select(0, rows_t).cpu().numpy().astype(np.float64)
        bad = np.abs(got - C_ref) > TOL * BND
        assert not bad.any(), f"{name} {point}: {int(bad.sum())} sampled elements out of tolerance"


# the configurations bench.py ends up timing on the large workloads, and one point of each other family
WHOLE_RESULT_CONFIGS = {
    "stencil27": [dict(point=(1, "serial", "row_split")), dict(point=(8, "parallel", "row_split")),
                  dict(point=(16, "serial", "nnz_balanced")), dict(point=(16, "parallel", "nnz_balanced")),
                  dict(point=(8, "parallel", "row_split"), reduce_size=2), dict(point=(4, "serial", "row_split"), block_size=512)],
    "rmat": [dict(point=(32, "serial", "nnz_balanced")), dict(point=(16, "serial", "nnz_balanced")),
             dict(point=(8, "parallel", "row_split")),
             dict(point=(1, "serial", "row_split")), dict(point=(16, "parallel", "nnz_balanced")),
             dict(point=(8, "parallel", "row_split"), long_row_min=1024), dict(point=(16, "parallel", "row_split"), reduce_size=8)],
    "skewed": [dict(point=(1, "serial", "row_split"), long_row_min=1024, wave_rows=1),
               dict(point=(4, "serial", "row_split"), long_row_min=1024),
               dict(point=(4, "parallel", "row_split"), long_row_min=4096, window_kb=2048),
               dict(point=(64, "serial", "nnz_balanced")), dict(point=(16, "parallel", "nnz_balanced")),
               dict(point=(4, "parallel", "row_split")), dict(point=(8, "serial", "row_split"), wave_rows=1)],
}


@pytest.mark.parametrize("name", ["stencil27", "rmat", "skewed"])
def test_full_size_every_element(name):
    # the oracle does a whole large workload in well under a second per pass on 16 threads; its result and bound
    # are taken block of rows by block of rows (a slice of the CSR arrays is a CSR matrix) to bound host memory
    # (operands and the first configuration's C packed into one allocation, as bench.py lays them out)
    p = wl.make_problem(name)
    dp = DeviceProblem(p, arena=True)
    outs = []
    for spec in WHOLE_RESULT_CONFIGS[name]:
        spec = dict(spec)
        cfg = binding.make_config(*spec.pop("point"), **spec)
        print("  config", binding.STRATEGY_NAMES[cfg.strategy], binding.SCHEDULE_NAMES[cfg.schedule], cfg.as_dict(), flush=True)
        outs.append((cfg, dp.run_cfg(cfg)))
    block = 1 << 17
    for r0 in range(0, p.M, block):
        r1 = min(p.M, r0 + block)
        lo, hi = int(p.rowptr[r0]), int(p.rowptr[r1])
        C_ref, BND = oracle.spmm_csr(r1 - r0, p.K, p.N, p.rowptr[r0:r1 + 1] - p.rowptr[r0], p.colidx[lo:hi],
                                     p.vals[lo:hi], p.B, nthreads=16)
        ref_t, bnd_t = torch.from_numpy(C_ref).cuda(), torch.from_numpy(BND).cuda()
        for cfg, C in outs:
            got = C[r0:r1].double()
            assert not torch.isnan(got).any(), f"{name} {cfg.as_dict()}: element never written in rows {r0}..{r1}"
            bad = (got - ref_t).abs() > TOL * bnd_t
            assert not bool(bad.any()), f"{name} {cfg.as_dict()}: {int(bad.sum())} elements of rows {r0}..{r1} out of tolerance"
        del ref_t, bnd_t


@pytest.mark.parametrize("name", ["stencil27", "rmat"])
def test_full_size_reduce_width_below_group_size(name):
    # a few {<1/g row, c col>, r} points with r < g at full size
    p = wl.make_problem(name)
    dp = DeviceProblem(p)
    rows = sample_rows(p)
    C_ref, BND = oracle.spmm_csr_rows(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, rows)
    rows_t = torch.from_numpy(rows).cuda()
    C = torch.empty((p.M, p.N), dtype=torch.float32, device="cuda:0")
    for g, r in [(4, 2), (8, 1), (32, 8), (64, 16)]:
        print("  g, r", g, r, flush=True)
        C.fill_(float("nan"))
        dp.launch_gr(C, g, r)
        torch.cuda.synchronize()
        assert not torch.isnan(C).any(), f"{name} g={g} r={r}: element never written"
        got = C.index_select(0, rows_t).cpu().numpy().astype(np.float64)
        bad = np.abs(got - C_ref) > TOL * BND
        assert not bad.any(), f"{name} g={g} r={r}: {int(bad.sum())} sampled elements out of tolerance"


@pytest.mark.parametrize("name", ["stencil27", "rmat", "skewed"])
def test_full_size_sddmm_every_entry(name):
    # the SDDMM oracle is fast enough to check every stored entry at full size
    p = wl.make_problem(name)
    X1 = wl.sddmm_left_operand(p)
    ref, bnd = oracle.sddmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, X1, p.B, nthreads=16)
    dp = DeviceProblem(p)
    X1d = torch.from_numpy(X1).cuda()
    ref_t = torch.from_numpy(ref).cuda()
    bnd_t = torch.from_numpy(bnd).cuda()
    for st in ("parallel", "serial"):
        for g in binding.GROUP_SIZES:
            print("  sddmm point", g, st, flush=True)
            out = dp.run_sddmm(X1d, g, st)
            assert not torch.isnan(out).any(), f"{name} sddmm g={g} {st}: entry never written"
            bad = (out.double() - ref_t).abs() > TOL * bnd_t
            assert not bool(bad.any()), f"{name} sddmm g={g} {st}: {int(bad.sum())} entries out of tolerance"


def test_twenty_million_short_rows():
    # many rows, few entries each, four dense columns: grids of more than a million workgroups,
    # row and entry counts far beyond 16 bits, C of 320 MB written four bytes per lane
    M, K, N = 20_000_000, 1000, 4
    rng = np.random.default_rng(77)
    lengths = rng.integers(0, 4, size=M)
    lengths[rng.integers(0, M, size=50)] = 900  # a few rows that span many tiles
    rowptr, colidx = wl.csr_from_lengths(rng, lengths.astype(np.int64), K)
    vals = wl.fill_values(rng, colidx.size, True)
    B = wl.fill_values(rng, K * N, True).reshape(K, N)
    p = wl.SpmmProblem("many_rows", M, K, N, rowptr, colidx, vals, B)
    print(p.row_stats(), flush=True)
    rows = sample_rows(p, n_random=5000)
    C_ref, _ = oracle.spmm_csr_rows(M, K, N, rowptr, colidx, vals, B, rows)
    dp = DeviceProblem(p)
    rows_t = torch.from_numpy(rows).cuda()
    C = torch.empty((M, N), dtype=torch.float32, device="cuda:0")
    for point in [(1, "serial", "row_split"), (4, "parallel", "row_split"), (64, "parallel", "row_split"),
                  (8, "serial", "nnz_balanced"), (64, "serial", "nnz_balanced"), (16, "parallel", "nnz_balanced"),
                  (1, "parallel", "nnz_balanced")]:
        print("  point", point, flush=True)
        dp.run(*point, C=C)
        assert not torch.isnan(C).any(), f"{point}: element never written"
        got = C.index_select(0, rows_t).cpu().numpy().astype(np.float64)
        assert np.array_equal(got, C_ref), f"{point}: {int((got != C_ref).sum())} sampled elements differ"


def test_two_billion_stored_entries():
    # positions close to the end of the int32 range: 2,000,000 rows of 1,024 entries = 2,048,000,000 entries
    # (16 GB of columns and values, made on the device from a formula the host can repeat for sampled rows)
    M, per_row, K, N = 2_000_000, 1024, 4096, 32
    nnz = M * per_row
    assert nnz < 2**31 - 65536
    dev = torch.device("cuda:0")
    if torch.cuda.get_device_properties(dev).total_memory < 40 * 2**30:
        pytest.skip("needs 40 GB of device memory")
    rowptr = (torch.arange(M + 1, dtype=torch.int64, device=dev) * per_row).to(torch.int32)
    pos = torch.arange(nnz, dtype=torch.int64, device=dev)
    colidx = ((pos // per_row) * 7 + (pos % per_row) * 13).remainder_(K).to(torch.int32)
    vals = ((pos // per_row + pos % per_row).remainder_(5) - 2).to(torch.float32)
    del pos
    rng = np.random.default_rng(5)
    B = wl.fill_values(rng, K * N, True).reshape(K, N)
    Bd = torch.from_numpy(B).to(dev)
    rows = np.unique(np.concatenate([rng.integers(0, M, size=300), [0, 1, M - 2, M - 1]]))
    j = np.arange(per_row)
    C_ref = np.zeros((rows.size, N))
    for n, r in enumerate(rows):
        cols = (r * 7 + j * 13) % K
        v = ((r + j) % 5 - 2).astype(np.float64)
        C_ref[n] = v @ B[cols].astype(np.float64)
    rows_t = torch.from_numpy(rows).to(dev)
    C = torch.empty((M, N), dtype=torch.float32, device=dev)
    for point in [(1, "serial", "row_split"), (16, "parallel", "row_split"), (16, "serial", "nnz_balanced"),
                  (64, "serial", "nnz_balanced"), (8, "parallel", "nnz_balanced")]:
        print("  point", point, flush=True)
        C.fill_(float("nan"))
        binding.sgap_spmm_csr_ex(M, K, N, rowptr, colidx, vals, Bd, C, point[0], binding.STRATEGIES[point[1]],
                                 binding.SCHEDULES[point[2]])
        torch.cuda.synchronize()
        assert not torch.isnan(C).any(), f"{point}: element never written"
        got = C.index_select(0, rows_t).cpu().numpy().astype(np.float64)
        assert np.array_equal(got, C_ref), f"{point}: {int((got != C_ref).sum())} sampled elements differ"
    # the SDDMM on the same pattern, one point
    X1 = torch.from_numpy(wl.fill_values(rng, 64 * N, True).reshape(64, N)).to(dev).repeat(M // 64, 1).contiguous()
    out = torch.full((nnz,), float("nan"), dtype=torch.float32, device=dev)
    binding.sgap_sddmm_csr(M, K, N, rowptr, colidx, vals, X1, Bd, out, 8, binding.STRATEGIES["parallel"])
    torch.cuda.synchronize()
    assert not torch.isnan(out).any()
    X1h = X1[:64].cpu().numpy().astype(np.float64)
    outh = out.view(M, per_row).index_select(0, rows_t).cpu().numpy().astype(np.float64)
    for n, r in enumerate(rows):
        cols = (r * 7 + j * 13) % K
        v = ((r + j) % 5 - 2).astype(np.float64)
        ref = v * (B[cols].astype(np.float64) @ X1h[r % 64])
        assert np.array_equal(outh[n], ref), f"sddmm row {r}"
