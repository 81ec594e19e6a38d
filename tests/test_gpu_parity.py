"""GPU parity: every (group_size, strategy, schedule) point of the HIP path
against the CPU oracle, through the C ABI, element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2209_02882_amd import binding
from paper_2209_02882_amd import workloads as wl

from gpu_util import GR_POINTS, POINTS, DeviceProblem, assert_close, full_reference, sample_rows

pytestmark = pytest.mark.gpu


def ids(pt):
    return f"g{pt[0]}-{pt[1]}-{pt[2]}"


# ---------------------------------------------------------------- primitives

def test_group_tree_sum_every_layout():
    rng = np.random.default_rng(1)
    for g in binding.GROUP_SIZES:
        lc = 1
        while g * lc <= 64:
            x = rng.integers(-8, 9, size=64).astype(np.float32)  # exact in fp32
            out = torch.full((64,), float("nan"), device="cuda:0")
            binding.sgap_debug_group_reduce(torch.from_numpy(x).cuda(), out, g, lc)
            got = out.cpu().numpy()
            want = np.zeros(64, np.float32)
            for lane in range(64):
                member = (lane // lc) % g
                if member == 0:
                    want[lane] = sum(x[lane + m * lc] for m in range(g))
            assert np.array_equal(got, want), f"group {g}, lanes per row {lc}"
            lc *= 2


def test_group_partial_sum_every_layout_and_width():
    rng = np.random.default_rng(11)
    for g in binding.GROUP_SIZES:
        lc = 1
        while g * lc <= 64:
            for r in [x for x in binding.GROUP_SIZES if x <= g]:
                x = rng.integers(-8, 9, size=64).astype(np.float32)
                out = torch.full((64,), float("nan"), device="cuda:0")
                binding.sgap_debug_group_partial_reduce(torch.from_numpy(x).cuda(), out, g, r, lc)
                got = out.cpu().numpy()
                want = np.zeros(64, np.float32)
                for lane in range(64):
                    member = (lane // lc) % g
                    if member % r == 0:
                        want[lane] = sum(x[lane + m * lc] for m in range(r))
                assert np.array_equal(got, want), f"group {g}, reduce {r}, lanes per row {lc}"
            lc *= 2


def test_group_seg_sum_every_layout_and_random_runs():
    rng = np.random.default_rng(2)
    for g in binding.GROUP_SIZES:
        lc = 1
        while g * lc <= 64:
            for trial in range(4):
                x = rng.integers(-8, 9, size=64).astype(np.float32)
                # random run boundaries per (slot, chunk): key changes with prob 0.4
                span = np.zeros(64, np.int32)
                want = np.zeros(64, np.float32)
                for lane in range(64):
                    chunk = lane % lc
                    slot = lane // (g * lc)
                    # runs are defined per slot, shared by its chunk lanes
                    r = np.random.default_rng(1000 * trial + 64 * g + slot)
                    cuts = r.random(g) < 0.4
                    member = (lane // lc) % g
                    s = 0
                    while member + s + 1 < g and not cuts[member + s + 1]:
                        s += 1
                    span[lane] = s
                    base = slot * g * lc + chunk
                    want[lane] = sum(x[base + (member + j) * lc] for j in range(s + 1))
                out = torch.full((64,), float("nan"), device="cuda:0")
                binding.sgap_debug_group_seg_reduce(torch.from_numpy(x).cuda(), torch.from_numpy(span).cuda(),
                                                    out, g, lc)
                got = out.cpu().numpy()
                # only the first lane of a run is used by the kernels, but every
                # lane's value is defined; check them all
                assert np.array_equal(got, want), f"group {g}, lanes per row {lc}, trial {trial}"
            lc *= 2


# ---------------------------------------------------- small named workloads

@pytest.fixture(scope="module")
def small_problems():
    out = {}
    for name, kw in [("uniform10", {}), ("uniform10_int", {}), ("powerlaw", {}),
                     ("stencil27", dict(scale_down=64)), ("rmat", dict(scale_down=64)),
                     ("skewed", dict(scale_down=25, N=64))]:
        p = wl.make_problem(name, **kw)
        out[name] = (DeviceProblem(p), full_reference(p))
    return out


@pytest.mark.parametrize("point", POINTS, ids=ids)
@pytest.mark.parametrize("name", ["uniform10", "uniform10_int", "powerlaw", "stencil27", "rmat", "skewed"])
def test_named_workloads_all_points(small_problems, name, point):
    dp, (C_ref, BND) = small_problems[name]
    C = dp.run(*point)
    assert_close(C, C_ref, BND, exact=name.endswith("_int"), what=f"{name} {ids(point)}")


def test_integer_variants_are_exact_everywhere():
    # integer-valued copies of the irregular workloads: every order of
    # summation gives the same fp32 number, so all points must agree exactly
    for name, kw in [("powerlaw", dict(scale_down=4)), ("skewed", dict(scale_down=25, N=32))]:
        p = wl.make_problem(name, **kw)
        rng = np.random.default_rng(5)
        p.vals = wl.fill_values(rng, p.nnz, True)
        p.B = wl.fill_values(rng, p.K * p.N, True).reshape(p.K, p.N)
        dp = DeviceProblem(p)
        C_ref, BND = full_reference(p)
        for point in POINTS:
            assert_close(dp.run(*point), C_ref, BND, exact=True, what=f"{name}-int {ids(point)}")


def test_operands_packed_into_one_allocation():
    # bench.py's layout: rowptr, colidx, vals, B and C one after the other in one allocation at 512-byte
    # boundaries (none of them on a page boundary of its own); the first output is the allocation's own C
    for name, kw in [("powerlaw", {}), ("rmat", dict(scale_down=64))]:
        p = wl.make_problem(name, **kw)
        dp = DeviceProblem(p, arena=True)
        C_ref, BND = full_reference(p)
        C = dp.new_output()
        assert C.data_ptr() == dp.B.data_ptr() + (p.K * p.N * 4 + 511) // 512 * 512
        for point in POINTS:
            assert_close(dp.run(*point, C=C), C_ref, BND, what=f"{name} packed {ids(point)}")
        cfg = binding.make_config(4, "serial", "row_split", long_row_min=64)
        assert_close(dp.run_cfg(cfg, C=C), C_ref, BND, what=f"{name} packed, window path")


def test_atomic_paths_repeat_within_tolerance():
    p = wl.make_problem("powerlaw", scale_down=2)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for _ in range(5):
        for point in [(8, "parallel", "nnz_balanced"), (32, "serial", "nnz_balanced")]:
            assert_close(dp.run(*point), C_ref, BND, what=ids(point))


# ---------------------------------------------------------------- edge cases

def csr_problem(name, M, K, N, lengths, seed, integer=False):
    rng = np.random.default_rng(seed)
    rowptr, colidx = wl.csr_from_lengths(rng, np.asarray(lengths), K)
    vals = wl.fill_values(rng, colidx.size, integer)
    B = wl.fill_values(rng, K * N, integer).reshape(K, N)
    return wl.SpmmProblem(name, M, K, N, rowptr, colidx, vals, B)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 6, 12, 20, 100, 130, 256, 260, 515, 1028])
def test_column_counts_and_vector_widths(N):
    rng = np.random.default_rng(N)
    M, K = 301, 257
    lengths = rng.integers(0, 40, size=M)
    p = csr_problem("cols", M, K, N, lengths, seed=N, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for point in POINTS:
        assert_close(dp.run(*point), C_ref, BND, exact=True, what=f"N={N} {ids(point)}")


def test_empty_matrix_overwrites_with_zero():
    M, K, N = 77, 50, 36
    p = csr_problem("empty", M, K, N, np.zeros(M, np.int64), seed=1)
    dp = DeviceProblem(p)
    for point in POINTS:
        C = dp.run(*point)
        assert torch.equal(C, torch.zeros_like(C)), ids(point)
        C = dp.run(*point, nnz_hint=-1)
        assert torch.equal(C, torch.zeros_like(C)), ids(point)


def test_identity_returns_B():
    K, N = 1000, 32
    p = wl.SpmmProblem("eye", K, K, N, np.arange(K + 1, dtype=np.int32), np.arange(K, dtype=np.int32),
                       np.ones(K, np.float32), wl.dense_operand(3, K, N, False))
    dp = DeviceProblem(p)
    for point in POINTS:
        C = dp.run(*point)
        assert torch.equal(C, dp.B), ids(point)


@pytest.mark.parametrize("lengths", [
    [5000],                                  # one long row
    [0, 0, 0, 3000, 0, 0],                   # long row between empty rows
    [1] * 2048,                              # every row one entry
    [64] * 64,                               # rows exactly one group wide
    [63, 1, 64, 65, 0, 127, 128, 129],       # rows around group boundaries
    [1023, 1, 1024, 1025, 0, 0, 2047, 1],    # rows around tile boundaries
    [0] * 3000 + [7] + [0] * 3000 + [2000],  # many empty rows in a tile window
    [2] * 512 + [0] * 5000 + [3] * 700,      # long empty stretch mid-matrix
    [1, 0] * 500 + [3] * 100,                # a tile's window: 1,000 rows, every other one without entries
    [0, 1, 0, 0, 2] * 300,                   # 1,024 entries span 1,700 rows, the rows with entries scattered among them
    [0] * 10 + [1, 1, 0] * 340 + [0] * 10,   # rows without entries first, last and in between
    [1] * 1024 + [0] + [1] * 1024 + [0] * 2, # a row without entries exactly where a tile ends
])
def test_row_shapes_at_boundaries(lengths):
    M = len(lengths)
    p = csr_problem("shape", M, 6000, 8, lengths, seed=M, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for point in POINTS:
        assert_close(dp.run(*point), C_ref, BND, exact=True, what=ids(point))
        assert_close(dp.run(*point, nnz_hint=-1), C_ref, BND, exact=True, what=ids(point) + " no hint")


def test_unsorted_and_duplicate_columns():
    rng = np.random.default_rng(12)
    M, K, N = 200, 64, 16
    lengths = rng.integers(0, 90, size=M)
    rowptr = np.zeros(M + 1, np.int32)
    rowptr[1:] = np.cumsum(lengths)
    colidx = rng.integers(0, K, size=rowptr[-1]).astype(np.int32)  # unsorted, with repeats
    p = wl.SpmmProblem("dups", M, K, N, rowptr, colidx, wl.fill_values(rng, colidx.size, True),
                       wl.fill_values(rng, K * N, True).reshape(K, N))
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for point in POINTS:
        assert_close(dp.run(*point), C_ref, BND, exact=True, what=ids(point))


def test_unaligned_operands_fall_back_to_narrow_vectors():
    rng = np.random.default_rng(13)
    M, K, N = 150, 90, 8
    p = csr_problem("unaligned", M, K, N, rng.integers(0, 30, size=M), seed=13, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for off in (1, 2):  # 4-byte and 8-byte aligned views
        Bbuf = torch.zeros(K * N + 4, device="cuda:0")
        Cbuf = torch.full((M * N + 4,), float("nan"), device="cuda:0")
        Bv = Bbuf[off:off + K * N]
        Bv.copy_(dp.B.reshape(-1))
        Cv = Cbuf[off:off + M * N]
        for point in POINTS:
            Cv.fill_(float("nan"))
            binding.sgap_spmm_csr_ex(M, K, N, dp.rowptr, dp.colidx, dp.vals, Bv, Cv, point[0],
                                     binding.STRATEGIES[point[1]], binding.SCHEDULES[point[2]])
            torch.cuda.synchronize()
            assert_close(Cv.reshape(M, N), C_ref, BND, exact=True, what=f"offset {off} {ids(point)}")
        assert torch.isnan(Cbuf[:off]).all() and torch.isnan(Cbuf[off + M * N:]).all()


def test_process_wide_schedule_entry_point():
    p = wl.make_problem("uniform10_int")
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    try:
        for sched in ("nnz_balanced", "row_split"):
            binding.sgap_set_schedule(binding.SCHEDULES[sched])
            for g in (1, 8, 64):
                for st in ("parallel", "serial"):
                    C = torch.full((p.M, p.N), float("nan"), device="cuda:0")
                    binding.sgap_spmm_csr(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C, g,
                                          binding.STRATEGIES[st])
                    torch.cuda.synchronize()
                    assert_close(C, C_ref, BND, exact=True, what=f"{sched} g{g} {st}")
    finally:
        binding.sgap_set_schedule(binding.SGAP_SCHED_ROW_SPLIT)


def test_runs_on_a_side_stream():
    p = wl.make_problem("uniform10_int")
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    s = torch.cuda.Stream()
    C = torch.full((p.M, p.N), float("nan"), device="cuda:0")
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        binding.sgap_spmm_csr_ex(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C, 8, 0, 1)
    s.synchronize()
    assert_close(C, C_ref, BND, exact=True)


def test_profile_hooks_count_main_kernels():
    p = wl.make_problem("uniform10")
    dp = DeviceProblem(p)
    binding.sgap_profile_enable(True)
    try:
        for _ in range(3):
            dp.run(8, "parallel", "nnz_balanced", poison=False)
        ms, n = binding.sgap_profile_collect()
        assert n == 3 and ms > 0
        assert binding.sgap_profile_collect() == (0.0, 0)
    finally:
        binding.sgap_profile_enable(False)


@pytest.mark.parametrize("n", [3, 1003 * 4 + 3, 4096 * 256 * 8 * 4, 4096 * 256 * 8 * 4 * 3 + 4 * 777 + 1])
def test_stream_kernels(n):
    # the copy moves every element (whole runs of eight accesses per lane, the rest of a workgroup's run, the last
    # elements that do not fill 16 bytes); the write-only kernel fills; the read-only one leaves its sink alone
    x = torch.arange(n, dtype=torch.float32, device="cuda:0")
    y = torch.zeros_like(x)
    binding.sgap_copy_f32(x, y)
    torch.cuda.synchronize()
    assert torch.equal(x, y)
    binding.sgap_stream_f32(None, y, n, 2)
    sink = torch.full((4,), 7.0, device="cuda:0")
    binding.sgap_stream_f32(x, sink, n, 1)
    torch.cuda.synchronize()
    assert bool((y == 1.0).all()) and bool((sink == 7.0).all())


def test_tuning_knobs_change_speed_not_results():
    p = wl.make_problem("stencil27", scale_down=64, N=128)
    rng = np.random.default_rng(3)
    p.vals = wl.fill_values(rng, p.nnz, True)
    p.B = wl.fill_values(rng, p.K * p.N, True).reshape(p.K, p.N)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    knobs = [(binding.SGAP_TUNE_TILE_COLS, v) for v in (0, 4, 30, 32, 64, 128, 1000)]
    knobs += [(binding.SGAP_TUNE_XCD_REMAP, v) for v in (0, 1, -1)]
    knobs += [(binding.SGAP_TUNE_ROWS_PER_GROUP, v) for v in (1, 3, 16, 0)]
    knobs += [(binding.SGAP_TUNE_PERSISTENT, v) for v in (1, 0)]
    try:
        for knob, value in knobs:
            binding.sgap_set_tuning(knob, value)
            for point in POINTS:
                if point[2] != "row_split":
                    continue
                assert_close(dp.run(*point), C_ref, BND, exact=True, what=f"knob {knob}={value} {ids(point)}")
    finally:
        binding.sgap_set_tuning(binding.SGAP_TUNE_TILE_COLS, 0)
        binding.sgap_set_tuning(binding.SGAP_TUNE_XCD_REMAP, -1)
        binding.sgap_set_tuning(binding.SGAP_TUNE_ROWS_PER_GROUP, 0)
        binding.sgap_set_tuning(binding.SGAP_TUNE_PERSISTENT, 0)
    with pytest.raises(binding.SgapError):
        binding.sgap_set_tuning(99, 1)


def test_per_call_configuration_knobs_change_speed_not_results():
    # the knobs of sgap_config one at a time on every point (those a point does not use are ignored)
    p = wl.make_problem("stencil27", scale_down=64, N=128)
    rng = np.random.default_rng(4)
    p.vals = wl.fill_values(rng, p.nnz, True)
    p.B = wl.fill_values(rng, p.K * p.N, True).reshape(p.K, p.N)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    knobs = [dict(block_size=v) for v in (128, 256, 512)] + [dict(tile_cols=v) for v in (4, 30, 64, 1000)]
    knobs += [dict(rows_per_group=v) for v in (1, 3, 16)] + [dict(xcd_remap=0), dict(persistent=1)]
    knobs += [dict(nnz_tile=v) for v in (256, 512, 2048)] + [dict(wave_rows=v) for v in (-1, 1)]
    knobs += [dict(block_size=128, tile_cols=256, rows_per_group=2), dict(block_size=512, wave_rows=1, persistent=1)]
    for kn in knobs:
        for point in POINTS:
            got = dp.run_cfg(binding.make_config(*point, **kn))
            assert_close(got, C_ref, BND, exact=True, what=f"{kn} {ids(point)}")


@pytest.mark.parametrize("N", [48, 64, 100, 128, 130, 256, 260, 520])
def test_serial_row_split_with_a_wavefront_per_row(N):
    # wave_rows = 1: the (column, value) pairs are the same for a whole wavefront; rows of every length
    # between empty and many runs of 64 entries, every group size (rows per wavefront)
    M, K = 1300, 3000
    rng = np.random.default_rng(N)
    lengths = rng.integers(0, 12, size=M)
    lengths[3::17] = rng.integers(60, 700, size=lengths[3::17].size)
    lengths[100:140] = 0
    lengths[-1] = 64
    p = csr_problem("mixed", M, K, N, lengths, seed=N, integer=True)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for g in binding.GROUP_SIZES:
        for block in (0, 512):  # (the layout has its own workgroup size: the knob is ignored)
            got = dp.run_cfg(binding.make_config(g, "serial", "row_split", wave_rows=1, block_size=block))
            assert_close(got, C_ref, BND, exact=True, what=f"N={N} g={g}")


def test_tuner_over_the_whole_space():
    p = wl.make_problem("skewed", scale_down=25, N=128)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    probe = binding.make_config(1, "serial", "row_split", long_row_min=1024)
    ws = dp.workspace_for(probe)
    for workspace in (None, ws):
        C = dp.new_output(poison=True)
        best, table = binding.sgap_autotune_csr_cfg(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C, reps=1,
                                                    workspace=workspace)
        torch.cuda.synchronize()
        assert_close(C, C_ref, BND, what="the fastest configuration's result is left in C")
        assert len(table) >= 28 + 21 and all(t.ms > 0 for t in table)
        assert best.ms == min(t.ms for t in table)
        windowed = [t for t in table if t.config.long_row_min > 0]
        assert bool(windowed) == (workspace is not None)
        # the configuration it returns runs as it is
        got = dp.run_cfg(best.config, workspace=workspace if best.config.long_row_min else None)
        assert_close(got, C_ref, BND, what=f"best configuration {best.config.as_dict()}")
    # the first 28 rated are the points of the narrow tuner, in its order
    assert [(t.config.group_size, t.config.strategy, t.config.schedule) for t in table[:28]] == \
        [(g, binding.STRATEGIES[st], binding.SCHEDULES[sc]) for g, st, sc in POINTS]


@pytest.mark.parametrize("name,kw", [("uniform10", {}), ("powerlaw", dict(scale_down=8)),
                                     ("stencil27", dict(scale_down=64)), ("skewed", dict(scale_down=25, N=64)),
                                     ("uniform10", dict(N=6)), ("uniform10", dict(N=7)), ("powerlaw", dict(scale_down=8, N=4))])
def test_reduce_width_below_group_size(name, kw):
    # {<1/g row, c col>, r} for every r < g: sub-group sums merged with atomics
    p = wl.make_problem(name, **kw)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for g, r in GR_POINTS:
        assert_close(dp.run_gr(g, r), C_ref, BND, what=f"{name} {kw} g={g} r={r}")
    # r = g is the plain-store point
    assert torch.equal(dp.run_gr(16, 16), dp.run(16, "parallel", "row_split"))
    rng = np.random.default_rng(17)
    p.vals = wl.fill_values(rng, p.nnz, True)
    p.B = wl.fill_values(rng, p.K * p.N, True).reshape(p.K, p.N)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    for g, r in GR_POINTS:
        assert_close(dp.run_gr(g, r), C_ref, BND, exact=True, what=f"{name} {kw} int g={g} r={r}")


def test_reduce_width_argument_checks():
    p = wl.make_problem("uniform10")
    dp = DeviceProblem(p)
    C = dp.new_output()
    for g, r in [(8, 16), (8, 3), (8, 0), (8, -1), (3, 1), (128, 8)]:
        with pytest.raises(binding.SgapError):
            dp.launch_gr(C, g, r)


def test_tuner_times_every_point_and_leaves_the_best_result():
    p = wl.make_problem("powerlaw", scale_down=4)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    C = dp.new_output(poison=True)
    best, table = binding.sgap_autotune_csr(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C, reps=2)
    torch.cuda.synchronize()
    got = [(t.group_size, binding.STRATEGY_NAMES[t.strategy], binding.SCHEDULE_NAMES[t.schedule]) for t in table]
    assert got == POINTS
    assert all(t.ms > 0 for t in table)
    assert best.ms == min(t.ms for t in table)
    assert (best.group_size, best.strategy, best.schedule) in [(t.group_size, t.strategy, t.schedule) for t in table]
    assert_close(C, C_ref, BND, what="result left by the tuner")


@pytest.mark.parametrize("name", ["powerlaw", "rmat", "skewed"])
def test_nnz_tile_sizes(name):
    # every tile size of the nnz-balanced serial kernel, on inputs with rows
    # far longer than a tile, rows without entries and many tiles per workgroup
    p = wl.make_problem(name, **{"powerlaw": dict(scale_down=2), "rmat": dict(scale_down=64),
                                 "skewed": dict(scale_down=25, N=64)}[name])
    rng = np.random.default_rng(5)
    p.vals = wl.fill_values(rng, p.nnz, True)
    p.B = wl.fill_values(rng, p.K * p.N, True).reshape(p.K, p.N)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    try:
        for tile in (256, 512, 1024, 2048, 0):
            binding.sgap_set_tuning(binding.SGAP_TUNE_NNZ_TILE, tile)
            for point in POINTS:
                if point[1:] != ("serial", "nnz_balanced"):
                    continue
                assert_close(dp.run(*point), C_ref, BND, exact=True, what=f"tile {tile} {ids(point)}")
    finally:
        binding.sgap_set_tuning(binding.SGAP_TUNE_NNZ_TILE, 0)
    with pytest.raises(binding.SgapError):
        binding.sgap_set_tuning(binding.SGAP_TUNE_NNZ_TILE, 300)


def test_wide_matrix_offsets_need_64_bits():
    # K*N*4 >= 2^32: the 32-bit offset fast path must not be taken
    K, N, M = 1 << 22, 256, 300
    rng = np.random.default_rng(21)
    lengths = rng.integers(0, 12, size=M)
    rowptr, colidx = wl.csr_from_lengths(rng, lengths, K)
    # make sure the far end of B is touched
    colidx[-1] = K - 1
    vals = wl.fill_values(rng, colidx.size, True)
    B = torch.zeros((K, N), dtype=torch.float32, device="cuda:0")
    rows_used = np.unique(colidx)
    Bsmall = wl.fill_values(rng, rows_used.size * N, True).reshape(-1, N)
    B[torch.from_numpy(rows_used.astype(np.int64)).cuda()] = torch.from_numpy(Bsmall).cuda()
    # oracle on a compacted copy (same rows of B, renumbered columns)
    remap = np.searchsorted(rows_used, colidx).astype(np.int32)
    C_ref, BND = oracle.spmm_csr(M, rows_used.size, N, rowptr, remap, vals, Bsmall)
    rp, ci, va = (torch.from_numpy(x).cuda() for x in (rowptr, colidx, vals))
    for point in POINTS:
        C = torch.full((M, N), float("nan"), device="cuda:0")
        binding.sgap_spmm_csr_ex(M, K, N, rp, ci, va, B, C, point[0], binding.STRATEGIES[point[1]],
                                 binding.SCHEDULES[point[2]])
        torch.cuda.synchronize()
        assert_close(C, C_ref, BND, exact=True, what=f"64-bit offsets {ids(point)}")


def test_calls_can_be_captured_in_a_graph_and_replayed():
    # after one eager call per point (the first call of a kernel instance asks
    # the runtime for its occupancy), the library only launches kernels on the
    # caller's stream: no allocation, no synchronisation, no memset nodes
    p = wl.make_problem("uniform10")
    rng = np.random.default_rng(9)
    p.vals = wl.fill_values(rng, p.nnz, True)
    p.B = wl.fill_values(rng, p.K * p.N, True).reshape(p.K, p.N)
    dp = DeviceProblem(p)
    C_ref, BND = full_reference(p)
    points = [(8, "parallel", "row_split"), (16, "serial", "nnz_balanced"), (4, "parallel", "nnz_balanced")]
    outs = [dp.new_output() for _ in points]
    for C, pt in zip(outs, points):
        dp.launch(C, *pt)  # eager warm-up
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for C, pt in zip(outs, points):
            dp.launch(C, *pt, stream=torch.cuda.current_stream())
    for replay in range(3):
        for C in outs:
            C.fill_(float("nan"))  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for C, pt in zip(outs, points):
            assert_close(C, C_ref, BND, exact=True, what=f"graph replay {replay} {ids(pt)}")


def test_validate_csr_counts_what_is_wrong():
    p = wl.make_problem("powerlaw", scale_down=8)
    rp = torch.from_numpy(p.rowptr).cuda()
    ci = torch.from_numpy(p.colidx).cuda()
    empty = int((np.diff(p.rowptr) == 0).sum())
    assert binding.sgap_validate_csr(p.M, p.K, rp, ci) == (0, 0, 0, empty)
    # columns out of range, on either side
    bad = ci.clone()
    bad[5] = -1
    bad[77] = p.K
    bad[78] = p.K + 5
    assert binding.sgap_validate_csr(p.M, p.K, rp, bad)[:2] == (0, 3)
    # a row whose columns are not ascending, and a repeated column
    long_row = int(np.argmax(np.diff(p.rowptr)))
    a = int(p.rowptr[long_row])
    uns = ci.clone()
    uns[a], uns[a + 1] = ci[a + 1].item(), ci[a].item()
    uns[a + 3] = uns[a + 2]
    assert binding.sgap_validate_csr(p.M, p.K, rp, uns) == (0, 0, 2, empty)
    # a damaged rowptr: one decreasing pair, a first entry that is not 0, a last entry that is not nnz
    rbad = rp.clone()
    rbad[10] = rbad[11] + 1
    assert binding.sgap_validate_csr(p.M, p.K, rbad, ci) == (2 if rbad[9] > rbad[10] else 1, 0, -1, -1)
    rbad = rp.clone()
    rbad[0] = 1 if p.rowptr[1] >= 1 else 0
    rbad[-1] += 1
    got = binding.sgap_validate_csr(p.M, p.K, rbad, ci)
    assert got[0] == (2 if p.rowptr[1] >= 1 else 1) and got[2:] == (-1, -1)
    # an empty matrix is fine
    z = torch.zeros(8, dtype=torch.int32, device="cuda:0")
    assert binding.sgap_validate_csr(7, 5, z, torch.zeros(0, dtype=torch.int32, device="cuda:0")) == (0, 0, 0, 7)
