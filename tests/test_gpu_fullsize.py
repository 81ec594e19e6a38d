"""Full-size workloads in the launch configuration the benchmark times,
checked on sampled output rows the oracle computes one by one, plus
properties that hold at any size (no element left unwritten)."""
import numpy as np
import pytest
import torch

import oracle
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
