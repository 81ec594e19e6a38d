"""The entry point for callers that cannot allocate (sgap_spmm_csr_cfg_static: working memory in an
array the library holds on the GPU) against sgap_spmm_csr_cfg with a caller-owned workspace, through
the C ABI: two calls in a row, the second on a smaller input, so that what the first call left in the
array must not leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2209_02882_amd import binding
from paper_2209_02882_amd import workloads as wl

from gpu_util import DeviceProblem, assert_close, full_reference
from test_gpu_panels import mixed_lengths
from test_gpu_parity import csr_problem

pytestmark = pytest.mark.gpu


def run_static(dp, cfg):
    p = dp.p
    C = dp.new_output(poison=True)
    binding.sgap_spmm_csr_cfg_static(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C, cfg)
    torch.cuda.synchronize()
    return C


@pytest.mark.parametrize("N", [64, 256])  # the claiming kernel / the owner wavefronts
def test_two_calls_in_a_row_the_second_smaller(N):
    # first: 1,400 long rows over many windows; second: a smaller matrix with fewer long rows and fewer windows
    first = csr_problem("first", 4200, 9000, N, mixed_lengths(4200, 9000, 41, long_every=3, long_len=(150, 900)),
                        seed=41, integer=True)
    second = csr_problem("second", 900, 2000, N, mixed_lengths(900, 2000, 42, long_every=7, long_len=(120, 500)),
                         seed=42, integer=True)
    for p, window_kb in ((first, 32), (second, 64)):
        dp = DeviceProblem(p)
        C_ref, BND = full_reference(p)
        for point in [(1, "serial", "row_split"), (8, "parallel", "row_split")]:
            cfg = binding.make_config(*point, long_row_min=100, window_kb=window_kb, max_long_rows=2048)
            with_workspace = dp.run_cfg(cfg)
            got = run_static(dp, cfg)
            # integer-valued inputs: both are exact, so they agree with the oracle and with each other
            assert_close(got, C_ref, BND, exact=True, what=f"{p.name} {point} built-in array")
            assert torch.equal(torch.nan_to_num(got), torch.nan_to_num(with_workspace))


def test_float_values_within_tolerance_of_both():
    p = csr_problem("mixed", 3000, 20000, 128, mixed_lengths(3000, 20000, 43, long_len=(1000, 6000)), seed=43)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    cfg = binding.make_config(4, "serial", "row_split", long_row_min=512, window_kb=256)
    for _ in range(2):
        assert_close(run_static(dp, cfg), C_ref, BND, what="float, built-in array")
    assert_close(dp.run_cfg(cfg), C_ref, BND, what="float, caller's workspace")


def test_sizes_beyond_the_array_are_refused_and_others_need_nothing():
    p = csr_problem("mixed", 500, 100000, 64, mixed_lengths(500, 100000, 44), seed=44, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    # 100,000 rows of B in windows of 1 KiB (4 rows): 511 windows, times a list of 8192 rows: 16 MB
    cfg = binding.make_config(1, "serial", "row_split", long_row_min=100, window_kb=1)
    assert binding.sgap_spmm_csr_workspace_size(p.M, p.K, p.N, cfg) > 8 << 20
    C = dp.new_output(poison=True)
    with pytest.raises(binding.SgapError) as err:
        binding.sgap_spmm_csr_cfg_static(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C, cfg)
    assert err.value.status == binding.SGAP_ERR_UNSUPPORTED and "8388608" in str(err.value)
    torch.cuda.synchronize()
    assert torch.isnan(C).all(), "a refused call must leave C untouched"
    cfg.max_long_rows = 1000  # now it fits
    assert_close(run_static(dp, cfg), C_ref, BND, exact=True, what="shorter list")
    # configurations without long rows set apart go straight through
    for point in [(8, "parallel", "row_split"), (16, "serial", "nnz_balanced")]:
        assert_close(run_static(dp, binding.make_config(*point)), C_ref, BND, exact=True, what=f"{point}")
