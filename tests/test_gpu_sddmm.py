"""GPU parity of the SDDMM kernels against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_02882_amd import binding
from paper_2209_02882_amd import workloads as wl

from gpu_util import TOL, DeviceProblem

pytestmark = pytest.mark.gpu

SDDMM_POINTS = [(g, st) for st in ("parallel", "serial") for g in binding.GROUP_SIZES]


def check(got, ref, bnd, exact, what):
    got = got.cpu().numpy().astype(np.float64)
    assert not np.isnan(got).any(), f"{what}: entries left unwritten"
    if exact:
        assert np.array_equal(got, ref), f"{what}: {np.count_nonzero(got != ref)} entries differ"
    else:
        bad = np.abs(got - ref) > TOL * bnd
        assert not bad.any(), f"{what}: {bad.sum()} entries outside {TOL} * bound"


@pytest.mark.parametrize("name,kw", [("uniform10", {}), ("uniform10_int", {}), ("powerlaw", dict(scale_down=8)),
                                     ("stencil27", dict(scale_down=64)), ("rmat", dict(scale_down=64)),
                                     ("skewed", dict(scale_down=25, N=64)),
                                     ("uniform10", dict(N=6)), ("uniform10", dict(N=7)), ("uniform10", dict(N=1)),
                                     ("powerlaw", dict(scale_down=8, N=260)), ("powerlaw", dict(scale_down=8, N=4))])
def test_every_point_matches_the_oracle(name, kw):
    p = wl.make_problem(name, **kw)
    X1 = wl.sddmm_left_operand(p)
    ref, bnd = oracle.sddmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, X1, p.B, nthreads=8)
    dp = DeviceProblem(p)
    X1d = torch.from_numpy(X1).cuda()
    try:
        for cache in (1, 0):  # with and without rows of X1 kept in registers
            binding.sgap_set_tuning(binding.SGAP_TUNE_SDDMM_ROW_CACHE, cache)
            for g, st in SDDMM_POINTS:
                if cache == 0 and st == "serial":
                    continue  # the knob only concerns the parallel strategy
                check(dp.run_sddmm(X1d, g, st), ref, bnd, name.endswith("_int"),
                      f"{name} {kw} g={g} {st} row cache {cache}")
    finally:
        binding.sgap_set_tuning(binding.SGAP_TUNE_SDDMM_ROW_CACHE, 1)


@pytest.mark.parametrize("name,kw", [("powerlaw", dict(scale_down=4)), ("rmat", dict(scale_down=64)),
                                     ("skewed", dict(scale_down=25, N=32))])
def test_integer_inputs_are_exact(name, kw):
    p = wl.make_problem(name, **kw)
    rng = np.random.default_rng(41)
    p.vals = wl.fill_values(rng, p.nnz, True)
    p.B = wl.fill_values(rng, p.K * p.N, True).reshape(p.K, p.N)
    X1 = wl.fill_values(rng, p.M * p.N, True).reshape(p.M, p.N)
    ref, bnd = oracle.sddmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, X1, p.B, nthreads=8)
    dp = DeviceProblem(p)
    X1d = torch.from_numpy(X1).cuda()
    for g, st in SDDMM_POINTS:
        check(dp.run_sddmm(X1d, g, st), ref, bnd, True, f"{name} int g={g} {st}")


def test_edge_shapes():
    dev = "cuda:0"
    # a matrix without entries, J = 0, one entry, a last tile of one entry, unknown nnz
    for M, K, J, lengths in [(5, 4, 8, [0, 0, 0, 0, 0]), (3, 3, 0, [1, 2, 0]), (1, 1, 3, [1]),
                             (1025, 7, 5, [1] * 1025), (3000, 16, 12, None)]:
        rng = np.random.default_rng(M * 31 + J)
        if lengths is None:
            lengths = rng.integers(0, 4, size=M)
        rowptr = np.zeros(M + 1, np.int32)
        rowptr[1:] = np.cumsum(lengths)
        nnz = int(rowptr[-1])
        colidx = rng.integers(0, K, size=nnz).astype(np.int32)
        vals = wl.fill_values(rng, nnz, True)
        X1 = wl.fill_values(rng, M * J, True).reshape(M, J)
        X2T = wl.fill_values(rng, K * J, True).reshape(K, J)
        ref, _ = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T)
        t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
        for g, st in SDDMM_POINTS:
            for hint in (None, -1):
                out = torch.full((nnz,), float("nan"), device=dev)
                binding.sgap_sddmm_csr(M, K, J, t(rowptr), t(colidx), t(vals), t(X1), t(X2T), out, g,
                                       binding.STRATEGIES[st], nnz_hint=hint)
                torch.cuda.synchronize()
                assert np.array_equal(out.cpu().numpy().astype(np.float64), ref), (M, K, J, g, st, hint)


def test_long_runs_of_empty_rows_overflow_the_row_window():
    # > 1024 empty rows between stored entries: the tile is cut at row boundaries
    M, K, J = 20000, 50, 8
    rng = np.random.default_rng(77)
    lengths = np.zeros(M, np.int64)
    lengths[rng.choice(M, size=40, replace=False)] = rng.integers(1, 200, size=40)
    rowptr = np.zeros(M + 1, np.int32)
    rowptr[1:] = np.cumsum(lengths)
    nnz = int(rowptr[-1])
    colidx = rng.integers(0, K, size=nnz).astype(np.int32)
    vals = wl.fill_values(rng, nnz, True)
    X1 = wl.fill_values(rng, M * J, True).reshape(M, J)
    X2T = wl.fill_values(rng, K * J, True).reshape(K, J)
    ref, _ = oracle.sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T)
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
    for g, st in SDDMM_POINTS:
        out = torch.full((nnz,), float("nan"), device="cuda:0")
        binding.sgap_sddmm_csr(M, K, J, t(rowptr), t(colidx), t(vals), t(X1), t(X2T), out, g, binding.STRATEGIES[st])
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), ref), (g, st)


def test_unaligned_operands_take_the_narrow_loads():
    p = wl.make_problem("uniform10", N=8)
    X1 = wl.sddmm_left_operand(p)
    ref, bnd = oracle.sddmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, X1, p.B)
    dp = DeviceProblem(p)
    for shift in (1, 2):  # 4- and 8-byte aligned views
        buf = torch.zeros(p.M * p.N + 4, dtype=torch.float32, device="cuda:0")
        X1d = buf[shift:shift + p.M * p.N]
        X1d.copy_(torch.from_numpy(X1).reshape(-1))
        for g, st in SDDMM_POINTS:
            out = torch.full((p.nnz,), float("nan"), device="cuda:0")
            binding.sgap_sddmm_csr(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, X1d, dp.B, out, g,
                                   binding.STRATEGIES[st])
            torch.cuda.synchronize()
            check(out, ref, bnd, False, f"shift {shift} g={g} {st}")
