"""GPU parity of the row-split schedule with long rows taken window by window
(sgap_spmm_csr_cfg with long_row_min set and a caller-owned workspace;
sgap_sddmm_csr_windows), against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_02882_amd import binding
from paper_2209_02882_amd import workloads as wl

from gpu_util import TOL, DeviceProblem, assert_close, full_reference, sample_rows
from test_gpu_parity import csr_problem

pytestmark = pytest.mark.gpu

ROW_SPLIT_POINTS = [(g, st, "row_split") for st in ("parallel", "serial") for g in binding.GROUP_SIZES]


class Panels:
    """The threshold, window size and list capacity the tests below run with; run() takes a point through
    sgap_spmm_csr_cfg with these and a workspace of exactly the size the library asks for."""

    def __init__(self):
        self.knobs = dict(long_row_min=0, window_kb=0, max_long_rows=0)

    def __call__(self, min_len, window_kb=0, max_long_rows=0):
        self.knobs = dict(long_row_min=min_len, window_kb=window_kb, max_long_rows=max_long_rows)

    def config(self, g, st, sc, **more):
        return binding.make_config(g, st, sc, **self.knobs, **more)

    def run(self, dp, g, st, sc, C=None, **more):
        return dp.run_cfg(self.config(g, st, sc, **more), C=C)

    def sddmm(self, dp, X1d, g, st):
        return dp.run_sddmm_windows(X1d, g, st, **self.knobs)


@pytest.fixture
def panels():
    return Panels()


def mixed_lengths(M, K, seed, long_every=17, long_len=(200, 900)):
    rng = np.random.default_rng(seed)
    lengths = rng.integers(0, 12, size=M)
    idx = np.arange(3, M, long_every)
    lengths[idx] = rng.integers(long_len[0], min(long_len[1], K) + 1, size=idx.size)
    return lengths


@pytest.mark.parametrize("N", [4, 8, 32, 64, 128, 256, 260, 512])
def test_long_rows_by_windows_match_the_oracle(panels, N):
    M, K = 1500, 4000
    p = csr_problem("mixed", M, K, N, mixed_lengths(M, K, N), seed=N, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for window_kb in (0, 64, 1):  # one window, a few dozen, the maximum of 255
        panels(100, window_kb)
        for point in ROW_SPLIT_POINTS:
            assert_close(panels.run(dp, *point), C_ref, BND, exact=True, what=f"N={N} window {window_kb} KiB {point}")


def test_float_values_within_tolerance_and_repeatable_within_it(panels):
    M, K, N = 3000, 20000, 64
    p = csr_problem("mixed", M, K, N, mixed_lengths(M, K, 5, long_len=(1000, 6000)), seed=5)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    panels(512, 256)
    for _ in range(3):
        for point in [(1, "serial", "row_split"), (8, "parallel", "row_split")]:
            assert_close(panels.run(dp, *point), C_ref, BND, what=f"float {point}")


def test_thresholds_at_the_edges(panels):
    M, K, N = 700, 900, 32
    p = csr_problem("mixed", M, K, N, mixed_lengths(M, K, 7, long_len=(100, 100)), seed=7, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    # rows exactly at the threshold are long; a threshold above every row leaves all to the row-split kernel;
    # threshold 1 makes every non-empty row long
    for min_len in (100, 101, 1):
        panels(min_len, 16)
        for point in [(4, "parallel", "row_split"), (2, "serial", "row_split")]:
            assert_close(panels.run(dp, *point), C_ref, BND, exact=True, what=f"min_len={min_len} {point}")


def test_more_long_rows_than_the_list_holds_switches_the_path_off(panels):
    M, K, N = 9000, 300, 16  # every row is long under min_len = 2: more than the default list of 8192 holds
    p = csr_problem("many_long", M, K, N, np.full(M, 5), seed=3, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for cap in (0, 100, 8999, 9000, 20000):  # too short four times (9000 rows), then long enough twice
        panels(2, 4, cap)
        for point in [(4, "parallel", "row_split"), (8, "serial", "row_split")]:
            assert_close(panels.run(dp, *point), C_ref, BND, exact=True, what=f"list of {cap} rows {point}")


def test_many_long_rows_of_wide_operands_take_several_passes(panels):
    # 128 columns and more: every long row has one owner wavefront per die; 12,000 long rows are more than
    # the wavefronts of a die own in one pass, and more than are sorted by length
    M, K, N = 12500, 3000, 128
    lengths = np.full(M, 40)
    lengths[::25] = 3
    p = csr_problem("many_long_wide", M, K, N, lengths, seed=4, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    panels(40, 256, 16384)
    for point in [(1, "serial", "row_split"), (4, "parallel", "row_split")]:
        assert_close(panels.run(dp, *point), C_ref, BND, exact=True, what=f"many long rows {point}")


def test_unsorted_and_repeated_columns_still_add_up(panels):
    M, K, N = 400, 2000, 32
    p = csr_problem("mixed", M, K, N, mixed_lengths(M, K, 11), seed=11, integer=True)
    rng = np.random.default_rng(12)
    for i in range(M):
        a, b = p.rowptr[i], p.rowptr[i + 1]
        perm = rng.permutation(b - a)
        p.colidx[a:b] = p.colidx[a:b][perm]
        p.vals[a:b] = p.vals[a:b][perm]
        if b - a > 3:
            p.colidx[a + 2] = p.colidx[a]
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    panels(100, 8)
    for point in [(1, "parallel", "row_split"), (16, "parallel", "row_split"), (4, "serial", "row_split")]:
        assert_close(panels.run(dp, *point), C_ref, BND, exact=True, what=f"unsorted {point}")


def test_other_schedules_and_unaligned_operands_ignore_the_threshold(panels):
    M, K, N = 500, 1000, 30  # N % 4 != 0: narrower loads, the window path does not apply and needs no workspace
    p = csr_problem("mixed", M, K, N, mixed_lengths(M, K, 13), seed=13, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    panels(100, 8)
    for point in [(4, "parallel", "row_split"), (8, "serial", "nnz_balanced"), (8, "parallel", "nnz_balanced")]:
        assert binding.sgap_spmm_csr_workspace_size(p.M, p.K, p.N, panels.config(*point)) == 0
        assert_close(panels.run(dp, *point), C_ref, BND, exact=True, what=f"ignored {point}")
    with pytest.raises(binding.SgapError):
        dp.run_cfg(binding.make_config(4, "parallel", "row_split", long_row_min=-1))
    with pytest.raises(binding.SgapError):  # the knobs of earlier versions are gone
        binding.sgap_set_tuning(6, 1024)


def test_workspace_is_required_sized_and_private_to_a_call(panels):
    M, K, N = 1500, 4000, 64
    p = csr_problem("mixed", M, K, N, mixed_lengths(M, K, 31), seed=31, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    panels(100, 64, 2000)
    cfg = panels.config(1, "serial", "row_split")
    need = binding.sgap_spmm_csr_workspace_size(p.M, p.K, p.N, cfg)
    windows = -(-K // (64 * 1024 // (N * 4)))
    assert need == 256 + (4 * 2000 * (windows + 4) + 255) // 256 * 256
    C = dp.new_output(poison=True)
    for ws in (None, torch.empty(need - 1, dtype=torch.uint8, device="cuda:0")):
        with pytest.raises(binding.SgapError):
            dp.launch_cfg(C, cfg, ws)
    torch.cuda.synchronize()
    assert torch.isnan(C).all(), "a refused call must leave C untouched"
    # two calls in flight on two streams, each with its own workspace (and stale contents in both)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    spaces = [torch.full((need,), 0xAB, dtype=torch.uint8, device="cuda:0") for _ in streams]
    outs = [dp.new_output(poison=True) for _ in streams]
    torch.cuda.synchronize()
    for rep in range(3):
        for st, ws, out in zip(streams, spaces, outs):
            with torch.cuda.stream(st):
                dp.launch_cfg(out, cfg, ws, stream=st)
    torch.cuda.synchronize()
    for out in outs:
        assert_close(out, C_ref, BND, exact=True, what="concurrent calls with private workspaces")


@pytest.mark.parametrize("name", ["skewed", "rmat"])
def test_full_size_sampled_rows(panels, name):
    # skewed: 1 KB rows of B, one member per wavefront; rmat: 128-byte rows, eight members, hub rows of 86,000 entries
    p = wl.make_problem(name)
    dp = DeviceProblem(p)
    rows = sample_rows(p)
    C_ref, BND = oracle.spmm_csr_rows(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, rows)
    rows_t = torch.from_numpy(rows).cuda()
    C = torch.empty((p.M, p.N), dtype=torch.float32, device="cuda:0")
    panels(1024)
    for point in [(1, "parallel", "row_split"), (4, "parallel", "row_split"), (2, "serial", "row_split")]:
        print("  point", point, flush=True)
        panels.run(dp, *point, C=C)
        assert not torch.isnan(C).any(), f"{point}: element never written"
        got = C.index_select(0, rows_t).cpu().numpy().astype(np.float64)
        bad = np.abs(got - C_ref) > TOL * BND
        assert not bad.any(), f"{point}: {int(bad.sum())} sampled elements out of tolerance"


def test_the_window_path_can_be_captured_in_a_graph_and_replayed(panels):
    # the path only launches kernels on the caller's stream: the counters in its
    # workspace are cleared by a kernel, not by a memset node
    M, K, N = 1500, 4000, 64
    p = csr_problem("mixed", M, K, N, mixed_lengths(M, K, 21), seed=21, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    panels(100, 64)
    points = [(1, "serial", "row_split"), (8, "parallel", "row_split")]
    configs = [panels.config(*pt) for pt in points]
    spaces = [dp.workspace_for(cfg) for cfg in configs]
    outs = [dp.new_output() for _ in points]
    for C, cfg, ws in zip(outs, configs, spaces):
        dp.launch_cfg(C, cfg, ws)  # eager warm-up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for C, cfg, ws in zip(outs, configs, spaces):
            dp.launch_cfg(C, cfg, ws, stream=torch.cuda.current_stream())
    for replay in range(3):
        for C in outs:
            C.fill_(float("nan"))  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for C, pt in zip(outs, points):
            assert_close(C, C_ref, BND, exact=True, what=f"graph replay {replay} {pt}")


def test_wide_matrix_offsets_need_64_bits(panels):
    # K*N*4 >= 2^32: offsets into B do not fit 32 bits, in the window kernel as in the row-split kernel
    K, N, M = 1 << 22, 256, 300
    rng = np.random.default_rng(23)
    lengths = mixed_lengths(M, K, 23, long_every=29, long_len=(300, 2500))
    rowptr, colidx = wl.csr_from_lengths(rng, lengths, K)
    colidx[-1] = K - 1  # the far end of B is touched
    vals = wl.fill_values(rng, colidx.size, True)
    rows_used = np.unique(colidx)
    Bsmall = wl.fill_values(rng, rows_used.size * N, True).reshape(-1, N)
    B = torch.zeros((K, N), dtype=torch.float32, device="cuda:0")
    B[torch.from_numpy(rows_used.astype(np.int64)).cuda()] = torch.from_numpy(Bsmall).cuda()
    # oracle on a compacted copy (same rows of B, renumbered columns: the order inside a row is kept)
    remap = np.searchsorted(rows_used, colidx).astype(np.int32)
    C_ref, BND = oracle.spmm_csr(M, rows_used.size, N, rowptr, remap, vals, Bsmall)
    rp, ci, va = (torch.from_numpy(x).cuda() for x in (rowptr, colidx, vals))
    panels(256)
    for point in [(1, "serial", "row_split"), (8, "parallel", "row_split")]:
        C = torch.full((M, N), float("nan"), device="cuda:0")
        cfg = panels.config(*point)
        ws = torch.empty(binding.sgap_spmm_csr_workspace_size(M, K, N, cfg), dtype=torch.uint8, device="cuda:0")
        binding.sgap_spmm_csr_cfg(M, K, N, rp, ci, va, B, C, cfg, workspace=ws)
        torch.cuda.synchronize()
        assert_close(C, C_ref, BND, exact=True, what=f"64-bit offsets {point}")


# ---------------------------------------------------------------- SDDMM on the same path

SDDMM_POINTS = [(g, st) for st in ("parallel", "serial") for g in binding.GROUP_SIZES]


def sddmm_reference(p, X1):
    return oracle.sddmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, X1, p.B, nthreads=8)


def check_sddmm(panels, dp, X1d, ref, bnd, exact, what, points=SDDMM_POINTS):
    for g, st in points:
        got = panels.sddmm(dp, X1d, g, st).cpu().numpy().astype(np.float64)
        assert not np.isnan(got).any(), f"{what} g={g} {st}: entries left unwritten"
        if exact:
            assert np.array_equal(got, ref), f"{what} g={g} {st}: {np.count_nonzero(got != ref)} entries differ"
        else:
            bad = np.abs(got - ref) > TOL * bnd
            assert not bad.any(), f"{what} g={g} {st}: {bad.sum()} entries outside tolerance"


@pytest.mark.parametrize("J", [32, 36, 64, 100, 128, 256, 16, 260])
def test_sddmm_long_rows_by_windows_match_the_oracle(panels, J):
    # J = 16 and 260 lie outside the path's range: the plain kernels must run as if the knob were off
    M, K = 1200, 5000
    p = csr_problem("mixed", M, K, J, mixed_lengths(M, K, J + 1), seed=J + 1, integer=True)
    X1 = wl.fill_values(np.random.default_rng(J), M * J, True).reshape(M, J)
    ref, bnd = sddmm_reference(p, X1)
    dp = DeviceProblem(p)
    X1d = torch.from_numpy(X1).cuda()
    for window_kb in (0, 64, 1):
        panels(100, window_kb)
        check_sddmm(panels, dp, X1d, ref, bnd, True, f"J={J} window {window_kb} KiB")


def test_sddmm_window_path_float_values_and_edges(panels):
    M, K, J = 2500, 30000, 128
    p = csr_problem("mixed", M, K, J, mixed_lengths(M, K, 17, long_len=(900, 7000)), seed=17)
    X1 = wl.fill_values(np.random.default_rng(18), M * J, False).reshape(M, J)
    ref, bnd = sddmm_reference(p, X1)
    dp = DeviceProblem(p)
    X1d = torch.from_numpy(X1).cuda()
    for min_len in (900, 1, 100000):  # some rows, every non-empty row, no row
        panels(min_len, 512)
        check_sddmm(panels, dp, X1d, ref, bnd, False, f"min_len={min_len}", points=[(8, "parallel"), (1, "parallel"), (4, "serial")])
    # more long rows than the list holds: the path switches itself off
    M2 = 9000
    p2 = csr_problem("many_long", M2, 300, 32, np.full(M2, 5), seed=19, integer=True)
    X12 = wl.fill_values(np.random.default_rng(20), M2 * 32, True).reshape(M2, 32)
    ref2, bnd2 = sddmm_reference(p2, X12)
    panels(2, 4)
    check_sddmm(panels, DeviceProblem(p2), torch.from_numpy(X12).cuda(), ref2, bnd2, True, "overflow",
                points=[(4, "parallel"), (8, "serial")])


def test_sddmm_full_size_skewed_every_entry(panels):
    p = wl.make_problem("skewed")
    X1 = wl.sddmm_left_operand(p)
    ref, bnd = oracle.sddmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, X1, p.B, nthreads=16)
    dp = DeviceProblem(p)
    X1d = torch.from_numpy(X1).cuda()
    ref_t, bnd_t = torch.from_numpy(ref).cuda(), torch.from_numpy(bnd).cuda()
    panels(1024)
    for g, st in [(8, "parallel"), (16, "parallel"), (4, "serial")]:
        print("  sddmm point", g, st, flush=True)
        out = panels.sddmm(dp, X1d, g, st)
        assert not torch.isnan(out).any(), f"g={g} {st}: entry never written"
        bad = (out.double() - ref_t).abs() > TOL * bnd_t
        assert not bool(bad.any()), f"g={g} {st}: {int(bad.sum())} entries out of tolerance"


def test_ttm_over_long_fibers_through_the_window_path(panels):
    # TTM along the last index is SpMM over the stored fibers (sgap_ttm_csf is sgap_spmm_csr_ex on the fiber-level
    # arrays), so a tensor with long fibers takes the window path through sgap_spmm_csr_cfg on the same arrays
    from paper_2209_02882_amd.device import DeviceTensor3
    from test_gpu_tensor import tensor_from

    p = tensor_from(40, 300, 6000, 64, [5] * 40, [3, 900, 7, 2500, 1], 33, integer=True)
    ref, bnd = oracle.ttm_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, p.X2, nthreads=8)
    dt = DeviceTensor3(p)
    panels(500, 64)
    for point in [(1, "serial", "row_split"), (8, "parallel", "row_split")]:
        cfg = panels.config(*point)
        ws = torch.empty(binding.sgap_spmm_csr_workspace_size(p.fibers, p.L, p.J, cfg), dtype=torch.uint8, device="cuda:0")
        Yf = torch.full((p.fibers, p.J), float("nan"), device="cuda:0")
        binding.sgap_spmm_csr_cfg(p.fibers, p.L, p.J, dt.eptr, dt.eidx, dt.vals, dt.X2, Yf, cfg, workspace=ws)
        torch.cuda.synchronize()
        assert_close(Yf, ref, bnd, exact=True, what=f"ttm with windows {point}")
