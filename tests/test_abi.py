"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_2209_02882_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(headers=("sgap.h", "sgap_debug.h")):
    names = set()
    for header in headers:
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b(sgap_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_symbols_are_exported_and_bound():
    lib = binding.load()
    names = declared_symbols()
    assert "sgap_spmm_csr" in names and "sgap_spmm_csr_ex" in names
    for name in names:
        assert hasattr(lib, name), f"{name} declared in a header but not exported"
        assert name in binding.EXPORTS, f"{name} has no Python binding signature"
    assert sorted(binding.EXPORTS) == names


def test_application_header_holds_no_test_scaffolding():
    public = declared_symbols(("sgap.h",))
    assert not [n for n in public if n.startswith(("sgap_debug_", "sgap_profile_"))] and "sgap_copy_f32" not in public
    for name in ("sgap_spmm_csr_cfg", "sgap_spmm_csr_workspace_size", "sgap_autotune_csr_cfg", "sgap_sddmm_csr_windows"):
        assert name in public


def test_configuration_defaults_workspace_size_and_checks():
    lib = binding.load()
    c = binding.make_config(8, "parallel", "row_split")
    assert c.as_dict() == dict(schedule=0, strategy=0, group_size=8, reduce_size=0, block_size=0, tile_cols=0,
                               rows_per_group=0, xcd_remap=-1, persistent=0, nnz_tile=0, wave_rows=0, long_row_min=0,
                               window_kb=0, max_long_rows=0)
    assert lib.sgap_config_init(None) == binding.SGAP_ERR_INVALID_ARG
    size = binding.sgap_spmm_csr_workspace_size
    assert size(1000, 1000, 64, c) == 0  # long rows are not set apart
    c.long_row_min = 512
    # automatic window: 3072 KiB of B = 12288 rows of 64 columns -> 1 window over K = 1000; default list of 8192 rows
    assert size(1000, 1000, 64, c) == 256 + 4 * 8192 * (1 + 4)
    c.window_kb, c.max_long_rows = 16, 100
    assert size(1000, 1000, 64, c) == 256 + (4 * 100 * (16 + 4) + 255) // 256 * 256  # 64 rows per window -> 16 windows
    assert size(1000, 1000, 62, c) == 0  # needs 16-byte loads
    c.schedule = binding.SGAP_SCHED_NNZ_BALANCED
    assert size(1000, 1000, 64, c) == 0
    c.schedule = binding.SGAP_SCHED_ROW_SPLIT
    ptrs = (0x1000, 0x2000, 0x3000, 0x4000, 0x5000)
    # the path applies (fake pointers are 16-byte aligned) and no workspace comes with the call
    assert lib.sgap_spmm_csr_cfg(4, 4, 4, *ptrs, ctypes.byref(c), -1, None, 0, None) == binding.SGAP_ERR_INVALID_ARG
    assert b"workspace" in lib.sgap_last_error()
    assert lib.sgap_spmm_csr_cfg(4, 4, 4, *ptrs, ctypes.byref(c), -1, 0x7000, 64, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_spmm_csr_cfg(4, 4, 4, *ptrs, ctypes.byref(c), -1, 0x7010, 1 << 20, None) == binding.SGAP_ERR_INVALID_ARG
    assert b"aligned" in lib.sgap_last_error()
    assert lib.sgap_spmm_csr_cfg(4, 4, 4, *ptrs, None, -1, None, 0, None) == binding.SGAP_ERR_INVALID_ARG
    for field, bad in [("block_size", 64), ("block_size", 1024), ("tile_cols", -1), ("rows_per_group", -1),
                       ("xcd_remap", 2), ("nnz_tile", 300), ("long_row_min", -1), ("window_kb", -1),
                       ("max_long_rows", -1), ("max_long_rows", (1 << 20) + 1), ("reduce_size", 3),
                       ("reduce_size", 16), ("group_size", 3), ("strategy", 2), ("schedule", 2), ("wave_rows", 2)]:
        bad_c = binding.make_config(8, "parallel", "row_split")
        setattr(bad_c, field, bad)
        assert lib.sgap_spmm_csr_cfg(4, 4, 4, *ptrs, ctypes.byref(bad_c), -1, None, 0, None) == \
            binding.SGAP_ERR_INVALID_ARG, field
        assert lib.sgap_spmm_csr_workspace_size(4, 4, 4, ctypes.byref(bad_c)) == -1, field
    # reduce_size below group_size belongs to the row-split parallel point only
    for st, sc in [("serial", "row_split"), ("parallel", "nnz_balanced")]:
        bad_c = binding.make_config(8, st, sc, reduce_size=2)
        assert lib.sgap_spmm_csr_cfg(4, 4, 4, *ptrs, ctypes.byref(bad_c), -1, None, 0, None) == binding.SGAP_ERR_INVALID_ARG
    # the SDDMM twin
    sd = binding.sgap_sddmm_csr_workspace_size
    assert sd(1000, 64) == 256 + 4 * 8192 * (1 + 4)  # 2048 KiB windows: 8192 rows of 64 columns
    assert sd(1000, 16) == 0 and sd(1000, 260) == 0 and sd(1000, 66) == 0
    assert lib.sgap_sddmm_csr_workspace_size(-1, 64, 0, 0) == -1
    assert lib.sgap_sddmm_csr_windows(4, 4, 64, *ptrs, 0x6000, 8, 0, 10, 100, 0, 0, None, 0, None) == \
        binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_sddmm_csr_windows(4, 4, 64, *ptrs, 0x6000, 8, 0, 10, -1, 0, 0, None, 0, None) == \
        binding.SGAP_ERR_INVALID_ARG
    # the wide tuner checks its arguments before anything else
    best = binding.TunedPoint()
    pbest = ctypes.cast(ctypes.pointer(best), ctypes.c_void_p)
    assert lib.sgap_autotune_csr_cfg(4, 4, 4, *ptrs, -1, 1, None, 0, None, 0, None, None, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_autotune_csr_cfg(4, 4, 4, *ptrs, -1, 0, None, 0, None, 0, None, pbest, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_autotune_csr_cfg(4, 4, 4, *ptrs, -1, 1, None, 0, None, 5, None, pbest, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_autotune_csr_cfg(0, 4, 4, *ptrs, -1, 1, None, 0, None, 0, None, pbest, None) == binding.SGAP_ERR_INVALID_ARG


def test_version_and_status_strings():
    lib = binding.load()
    assert lib.sgap_version() >= 100
    assert lib.sgap_status_string(0) == b"ok"
    assert lib.sgap_status_string(1) == b"invalid argument"
    assert lib.sgap_status_string(77) == b"unknown status"


def test_schedule_selector():
    lib = binding.load()
    assert lib.sgap_get_schedule() == binding.SGAP_SCHED_ROW_SPLIT
    assert lib.sgap_set_schedule(binding.SGAP_SCHED_NNZ_BALANCED) == 0
    assert lib.sgap_get_schedule() == binding.SGAP_SCHED_NNZ_BALANCED
    assert lib.sgap_set_schedule(5) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_get_schedule() == binding.SGAP_SCHED_NNZ_BALANCED
    assert lib.sgap_set_schedule(binding.SGAP_SCHED_ROW_SPLIT) == 0


@pytest.mark.parametrize("kw,msg", [
    (dict(M=-1), b"negative"),
    (dict(N=-3), b"negative"),
    (dict(M=2**31 - 1), b"int32"),
    (dict(group=3), b"group_size"),
    (dict(group=0), b"group_size"),
    (dict(group=128), b"group_size"),
    (dict(strategy=2), b"strategy"),
    (dict(schedule=9), b"schedule"),
    (dict(nnz_hint=-5), b"nnz_hint"),
    (dict(rowptr=None), b"null"),
    (dict(C=None), b"null"),
    (dict(B=None), b"null"),
])
def test_invalid_arguments_are_rejected_without_launch(kw, msg):
    lib = binding.load()
    # fake non-null "device pointers": validation must fail before any use
    a = dict(M=4, K=4, N=4, rowptr=0x1000, colidx=0x2000, vals=0x3000, B=0x4000, C=0x5000,
             group=8, strategy=0, schedule=0, nnz_hint=-1)
    a.update(kw)
    rc = lib.sgap_spmm_csr_ex(a["M"], a["K"], a["N"], a["rowptr"], a["colidx"], a["vals"], a["B"], a["C"],
                              a["group"], a["strategy"], a["schedule"], a["nnz_hint"], None)
    assert rc == binding.SGAP_ERR_INVALID_ARG
    assert msg in lib.sgap_last_error()


def test_reduce_size_and_tuner_arguments_are_checked_without_launch():
    lib = binding.load()
    ptrs = (0x1000, 0x2000, 0x3000, 0x4000, 0x5000)
    for g, r in [(8, 16), (8, 3), (8, 0), (8, -2), (3, 1)]:
        assert lib.sgap_spmm_csr_gr(4, 4, 4, *ptrs, g, r, -1, None) == binding.SGAP_ERR_INVALID_ARG
    best = binding.PointTime()
    pbest = ctypes.cast(ctypes.pointer(best), ctypes.c_void_p)
    assert lib.sgap_autotune_csr(4, 4, 4, *ptrs, -1, 3, None, None, None) == binding.SGAP_ERR_INVALID_ARG
    assert b"best" in lib.sgap_last_error()
    assert lib.sgap_autotune_csr(4, 4, 4, *ptrs, -1, 0, None, pbest, None) == binding.SGAP_ERR_INVALID_ARG
    assert b"reps" in lib.sgap_last_error()
    assert lib.sgap_autotune_csr(0, 4, 4, *ptrs, -1, 1, None, pbest, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_set_tuning(binding.SGAP_TUNE_NNZ_TILE, 300) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_set_tuning(binding.SGAP_TUNE_NNZ_TILE, 0) == 0


def test_sddmm_arguments_are_checked_without_launch():
    lib = binding.load()
    ok = dict(M=4, K=4, J=4, rowptr=0x1000, colidx=0x2000, vals=0x3000, X1=0x4000, X2T=0x5000, out=0x6000,
              group=8, strategy=0, nnz_hint=-1)
    for kw, msg in [(dict(M=-1), b"negative"), (dict(J=-2), b"negative"), (dict(group=3), b"group_size"),
                    (dict(strategy=5), b"strategy"), (dict(nnz_hint=-7), b"nnz_hint"), (dict(rowptr=None), b"null"),
                    (dict(out=None, nnz_hint=5), b"null"), (dict(X1=None), b"null"), (dict(X2T=None), b"null")]:
        a = dict(ok)
        a.update(kw)
        rc = lib.sgap_sddmm_csr(a["M"], a["K"], a["J"], a["rowptr"], a["colidx"], a["vals"], a["X1"], a["X2T"],
                                a["out"], a["group"], a["strategy"], a["nnz_hint"], None)
        assert rc == binding.SGAP_ERR_INVALID_ARG, kw
        assert msg in lib.sgap_last_error(), kw
    # nothing to do: no rows, or no stored entries
    assert lib.sgap_sddmm_csr(0, 4, 4, None, None, None, None, None, None, 8, 0, -1, None) == 0
    assert lib.sgap_sddmm_csr(4, 4, 4, None, None, None, None, None, None, 8, 1, 0, None) == 0


def test_tensor_arguments_are_checked_without_launch():
    lib = binding.load()
    ok = dict(I=4, K=4, L=4, J=4, fptr=0x1000, fidx=0x2000, eptr=0x3000, eidx=0x4000, vals=0x5000, X1=0x6000,
              X2=0x7000, Y=0x8000, group=8, strategy=0)
    for kw, msg in [(dict(I=-1), b"negative"), (dict(J=-2), b"negative"), (dict(L=1 << 40), b"int32"),
                    (dict(group=3), b"group_size"), (dict(group=128), b"group_size"), (dict(strategy=5), b"strategy"),
                    (dict(fptr=None), b"null"), (dict(Y=None), b"null"), (dict(X1=None), b"null"),
                    (dict(X2=None), b"null")]:
        a = dict(ok)
        a.update(kw)
        rc = lib.sgap_mttkrp_csf(a["I"], a["K"], a["L"], a["J"], a["fptr"], a["fidx"], a["eptr"], a["eidx"],
                                 a["vals"], a["X1"], a["X2"], a["Y"], a["group"], a["strategy"], None)
        assert rc == binding.SGAP_ERR_INVALID_ARG, kw
        assert msg in lib.sgap_last_error(), kw
    # nothing to do: no slices, or no columns
    assert lib.sgap_mttkrp_csf(0, 4, 4, 4, None, None, None, None, None, None, None, None, 8, 0, None) == 0
    assert lib.sgap_mttkrp_csf(4, 4, 4, 0, None, None, None, None, None, None, None, None, 8, 1, None) == 0
    # TTM takes the SpMM checks with fibers as rows
    assert lib.sgap_ttm_csf(-1, 4, 4, None, None, None, None, None, 8, 0, 0, -1, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_ttm_csf(4, 4, 4, 0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 8, 0, 9, -1, None) \
        == binding.SGAP_ERR_INVALID_ARG
    assert b"schedule" in lib.sgap_last_error()
    assert lib.sgap_ttm_csf(0, 4, 4, None, None, None, None, None, 8, 0, 0, -1, None) == 0


def test_validate_arguments_are_checked_without_launch():
    lib = binding.load()
    report = (ctypes.c_int64 * 4)()
    assert lib.sgap_validate_csr(-1, 4, 0x1000, 0x2000, 3, report, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_validate_csr(4, 4, 0x1000, 0x2000, -3, report, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_validate_csr(4, 4, None, 0x2000, 3, report, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_validate_csr(4, 4, 0x1000, None, 3, report, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_validate_csr(4, 4, 0x1000, 0x2000, 3, None, None) == binding.SGAP_ERR_INVALID_ARG
    assert b"null" in lib.sgap_last_error()


def test_entry_counts_beyond_the_position_range_are_refused():
    lib = binding.load()
    ptrs = [0x1000 * i for i in range(1, 6)]
    assert lib.sgap_spmm_csr_ex(4, 4, 4, *ptrs, 8, 0, 0, 2**31 - 65535, None) == binding.SGAP_ERR_INVALID_ARG
    assert b"2^31" in lib.sgap_last_error()
    assert lib.sgap_sddmm_csr(4, 4, 4, 0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 8, 0, 2**31 - 1, None) \
        == binding.SGAP_ERR_INVALID_ARG


def test_empty_shapes_are_ok_without_launch():
    lib = binding.load()
    assert lib.sgap_spmm_csr_ex(0, 5, 8, None, None, None, None, None, 8, 0, 0, -1, None) == 0
    assert lib.sgap_spmm_csr_ex(5, 5, 0, None, None, None, None, None, 8, 1, 1, -1, None) == 0
    assert lib.sgap_spmm_csr(0, 0, 0, None, None, None, None, None, 64, 1, None) == 0


def test_debug_entry_points_validate_layout():
    lib = binding.load()
    assert lib.sgap_debug_group_reduce(0x1000, 0x2000, 16, 8, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_debug_group_reduce(None, 0x2000, 4, 4, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_debug_group_seg_reduce(0x1000, 0x2000, 0x3000, 3, 1, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_copy_f32(0x1001, 0x2000, 4, None) == binding.SGAP_ERR_INVALID_ARG
    assert lib.sgap_copy_f32(None, None, 0, None) == 0


def test_binding_refuses_cpu_tensors():
    import torch

    t = torch.zeros(4)
    with pytest.raises(TypeError):
        binding.sgap_copy_f32(t, t)


def tile_deal(lib, tiles, grid, block):
    cap = tiles + 1
    buf = (ctypes.c_int64 * cap)()
    n = lib.sgap_debug_tile_deal(tiles, grid, block, buf, cap)
    assert 0 <= n <= tiles
    return list(buf[:n])


@pytest.mark.parametrize("tiles,grid", [(0, 1), (1, 1), (7, 7), (8, 8), (9, 8), (100, 16), (1000, 1024), (1029, 1024),
                                        (4117, 1024), (48754, 1024), (25844, 1280), (777, 40), (5000, 1000), (333, 24)])
def test_every_tile_goes_to_exactly_one_workgroup(tiles, grid):
    lib = binding.load()
    seen = []
    per_die = {}
    by_die = grid >= 8 and grid % 8 == 0 and tiles > grid  # else plain round-robin
    for b in range(grid):
        mine = tile_deal(lib, tiles, grid, b)
        assert mine == sorted(mine), "a workgroup walks its tiles in ascending order"
        seen += mine
        per_die.setdefault(b % 8 if by_die else 0, []).extend(mine)
    assert sorted(seen) == list(range(tiles))
    if not by_die:
        assert all(tile_deal(lib, tiles, grid, b) == list(range(b, tiles, grid)) for b in range(grid))
    if tiles >= 8 * 64 and by_die:
        # every die gets an even share, in runs of neighbouring tiles
        sizes = [len(v) for v in per_die.values()]
        assert max(sizes) - min(sizes) <= max(1, tiles // 64)
        t = sorted(per_die[0])
        runs = 1 + sum(1 for x, y in zip(t, t[1:]) if y != x + 1)
        # chunks of about tiles/128 neighbouring tiles, at most one round of the die's workgroups
        chunk = max(1, min(tiles // 128, grid // 8))
        assert runs <= -(-tiles // chunk) // 8 + 1
    assert lib.sgap_debug_tile_deal(10, 4, 4, None, 0) == -1


def test_serial_plan_keeps_partial_sums_on_chip_and_fills_the_chip():
    lib = binding.load()

    def plan(g, lc, vec, nnz, cus=256, forced=0):
        tile, merge, lanes = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
        assert lib.sgap_debug_plan_nnz_serial(g, lc, vec, nnz, cus, forced, ctypes.byref(tile), ctypes.byref(merge),
                                              ctypes.byref(lanes)) == 0
        used.append(lanes.value)
        return tile.value, bool(merge.value)

    used = []

    # large matrices: 1024 or 2048 entries, shrunk until the slots fit 34 KB
    assert plan(32, 8, 4, 50_000_000) == (1024, True)
    assert plan(64, 1, 4, 50_000_000) == (2048, True)
    assert plan(8, 32, 4, 26_000_000) == (512, True)      # 128 columns: 65 slots of 520 bytes
    assert used[-1] == 32
    # small groups at wide N: most of the LDS at the smallest tile (129 slots of 520 bytes) ...
    assert plan(2, 32, 4, 26_000_000) == (256, True) and used[-1] == 32
    # ... and fewer chunk lanes per entry where even that is too little (257 slots: 1032 bytes each do not fit, 520 do)
    assert plan(1, 64, 4, 57_000_000) == (256, True) and used[-1] == 32
    assert plan(1, 64, 1, 57_000_000) == (1024, True) and used[-1] == 32   # 1025 slots of 136 bytes
    assert plan(2, 32, 4, 26_000_000, forced=256) == (256, False)          # a forced tile keeps the plain rule
    # small matrices: smaller tiles so that the chip's ~1024 resident workgroups all get work
    assert plan(16, 8, 4, 10_240)[0] == 256
    assert plan(16, 16, 4, 1_053_925)[0] in (256, 512)
    # unknown nnz, narrow loads or a forced size keep the base choice / the forced one
    assert plan(16, 8, 4, -1)[0] == 1024
    assert plan(16, 8, 2, 10_240)[0] == 1024
    assert plan(16, 8, 4, 10_240, forced=2048)[0] == 2048
    assert lib.sgap_debug_plan_nnz_serial(3, 8, 4, 0, 256, 0, None, None, None) == binding.SGAP_ERR_INVALID_ARG


def test_reordering_checks_its_arguments_on_the_host():
    lib = binding.load()
    size = lib.sgap_reorder_rows_workspace_size
    assert size(-1) == -1
    assert size(0) >= 256 and size(0) % 256 == 0
    # two int32 per row, the key counters and a sum per block of rows
    assert size(2_097_152) >= 8 * 2_097_152 + 8 * 4097 and size(2_097_152) % 256 == 0
    assert size(10) <= size(11) <= size(100_000)
    fake = ctypes.c_void_p(256)  # never dereferenced: every call below is refused before anything is launched
    bad = [
        dict(M=-1), dict(K=-1), dict(M=2**31), dict(order=2), dict(order=-1), dict(rowptr=None), dict(rowptr_out=None),
        dict(perm=None), dict(K=0), dict(workspace=None), dict(workspace_bytes=100), dict(workspace=ctypes.c_void_p(264)),
    ]
    for change in bad:
        a = dict(M=4, K=4, rowptr=fake, colidx=fake, vals=fake, order=0, perm=fake, rowptr_out=fake, colidx_out=fake,
                 vals_out=fake, workspace=fake, workspace_bytes=1 << 20)
        a.update(change)
        rc = lib.sgap_reorder_rows_csr(a["M"], a["K"], a["rowptr"], a["colidx"], a["vals"], a["order"], a["perm"],
                                       a["rowptr_out"], a["colidx_out"], a["vals_out"], a["workspace"],
                                       a["workspace_bytes"], None)
        assert rc == binding.SGAP_ERR_INVALID_ARG, change


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 without warnings,
    # and a C program must link against the built library (it is not run: no GPU here)
    import shutil
    import subprocess

    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_sgap.c"
    src.write_text(
        '#include "sgap.h"\n'
        '#include "sgap_debug.h"\n'
        "int main(void)\n{\n"
        "    float c[4];\n"
        "    sgap_config cfg;\n"
        "    int rc = sgap_spmm_csr(0, 0, 0, 0, 0, 0, 0, c, 8, SGAP_REDUCE_PARALLEL, 0);\n"
        "    rc |= sgap_config_init(&cfg);\n"
        "    rc |= sgap_spmm_csr_cfg(0, 0, 0, 0, 0, 0, 0, c, &cfg, -1, 0, 0, 0);\n"
        "    rc |= sgap_profile_enable(0);\n"
        "    return rc == SGAP_OK && sgap_version() >= 100 ? 0 : 1;\n"
        "}\n")
    inc = os.path.join(root, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-fsyntax-only", str(src)],
                   check=True)
    binding.load()  # raises if the library has not been built
    lib_dir = os.path.dirname(binding.LIB_PATH)
    exe = tmp_path / "use_sgap"
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", lib_dir, "-lsgap",
                    "-Wl,--unresolved-symbols=ignore-in-shared-libs"], check=True)
    assert exe.exists()
