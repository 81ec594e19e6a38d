#!/usr/bin/env python3
"""Benchmark of the CSR SpMM hot path on one MI355X.

A "step" is one whole SpMM call (row-zeroing pass included where the point
needs one) on a seeded synthetic workload that is resident in HBM.  All 28
(group_size, strategy, schedule) points are swept briefly; the best one is
then timed for exactly --steps steps and reported as ONE JSON line on stdout:
effective GFLOP/s = 2*nnz*N/t, with the HBM roofline of the main kernel
(minimal bytes nnz*8 + (M+1)*4 + K*N*4 + M*N*4 over its event-timed duration)
and the CPU oracle timed on the host next to it.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X published fp32 vector rate
# Rate at which 256 compute units deliver gathered dwordx4 operands that hit in
# L1, measured with paper_2209_02882_amd/microbench/gather_bandwidth.hip
# (profiles/microbenchmarks.md): 55-60 bytes per clock per compute unit.
L1_GATHER_TBS = 36.0

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE),
# scaled by the same counters on the library's plain copy kernel; keyed by
# (workload, group, strategy, schedule).  See profiles/ for the runs.
MEASURED_TRAFFIC_BYTES: dict = {
    ("stencil27", 1, "parallel", "row_split"): 2_287_184_383,   # profiles/row_split_kernel_stencil27.md
    ("stencil27", 1, "serial", "row_split"): 2_260_465_487,     # profiles/row_split_kernel_stencil27_serial.md
    ("rmat", 16, "serial", "nnz_balanced"): 4_398_701_021,      # profiles/nnz_serial_kernel_rmat.md (main kernel)
    ("skewed", 64, "serial", "nnz_balanced"): 59_904_989_739,   # profiles/nnz_serial_kernel_skewed.md (main kernel)
    ("powerlaw", 16, "serial", "nnz_balanced"): 242_820_253,    # profiles/nnz_serial_kernel_powerlaw.md (main kernel)
    # --long-row-min 1024: all five kernels of the call, profiles/panel_long_rows_kernel_skewed.md
    ("skewed", 4, "serial", "row_split", 1024): 7_695_174_915,
}


# the same for --op sddmm, keyed by (workload, group, strategy)
MEASURED_SDDMM_TRAFFIC_BYTES: dict = {
    ("stencil27", 8, "parallel"): 4_622_814_612,   # profiles/sddmm_rowcache_kernel_stencil27.md
    ("rmat", 8, "parallel"): 4_640_438_673,        # profiles/sddmm_rowcache_kernel_rmat.md
    # --long-row-min 1024: all five kernels of the call, profiles/panel_sddmm_kernel_skewed.md
    ("skewed", 16, "parallel", 1024): 8_349_418_150,
}


# the same for --op mttkrp / ttm, keyed by (op, workload, point...)
MEASURED_TENSOR_TRAFFIC_BYTES: dict = {
    ("mttkrp", "tensor3", 8, "parallel"): 1_744_923_312,   # profiles/mttkrp_kernel_tensor3.md
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_point(dp, torch, binding, C, point, iters):
    g, st, sc = point
    p = dp.p
    args = (p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C, g,
            binding.STRATEGIES[st], binding.SCHEDULES[sc])
    binding.sgap_spmm_csr_ex(*args)  # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        binding.sgap_spmm_csr_ex(*args)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / iters


def launch_stats(torch, launch, n, flush=None):
    """Per-launch durations in ms over n launches, timed with events on the
    stream the launches go to (torch's current stream, which is the stream the
    library is handed).  With `flush` (a tensor larger than every cache of the
    chip) the caches are overwritten before each launch."""
    evs = []
    for _ in range(n):
        if flush is not None:
            flush.add_(1.0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        launch()
        e1.record()
        evs.append((e0, e1))
    torch.cuda.synchronize()
    ms = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    return {"median": ms[len(ms) // 2], "min": ms[0], "launches": n}


def ceilings(p):
    """The three ceilings of a gather-reduce SpMM, as times for one launch: HBM
    at its published rate over the minimal bytes, the vector memory path
    delivering one operand per multiply-add (nnz*N*4 bytes) at the measured
    L1-hit gather rate, and the fp32 vector units."""
    return {
        "hbm_minimal_bytes_ms": p.minimal_bytes() / (HBM_PEAK_GBS * 1e9) * 1e3,
        "gather_l1_ms": p.nnz * p.N * 4 / (L1_GATHER_TBS * 1e12) * 1e3,
        "fp32_vector_ms": p.flops() / (FP32_VECTOR_PEAK_TFLOPS * 1e12) * 1e3,
    }


def cpu_baseline(p):
    """The oracle as it stands, timed on this host: all cores on the whole
    workload (static row split), and one core on the first quarter of the rows."""
    import oracle

    cores = len(os.sched_getaffinity(0))
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env))
    # all cores: the whole workload, repeated until about 10 s of wall time
    reps, t_all = 0, 0.0
    while t_all < 10.0 and reps < 200:
        t0 = time.perf_counter()
        oracle.spmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, p.B, nthreads=cores)
        t_all += time.perf_counter() - t0
        reps += 1
    # one core: the first quarter of the rows, once
    rows = max(1, p.M // 4)
    nnz_part = int(p.rowptr[rows])
    t0 = time.perf_counter()
    oracle.spmm_csr(rows, p.K, p.N, p.rowptr[:rows + 1], p.colidx[:nnz_part], p.vals[:nnz_part], p.B, nthreads=1)
    t_one = time.perf_counter() - t0
    return {
        "value": 2.0 * p.nnz * p.N * reps / t_all / 1e9,
        "unit": "GFLOP/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"whole {p.name} workload x{reps}, fp64 row-by-row oracle (result and error bound), "
                  f"static row split over {cores} threads, {t_all:.1f} s",
        "seconds_per_pass": t_all / reps,
        "single_thread_gflops": 2.0 * nnz_part * p.N / t_one / 1e9,
        "single_thread_sample": f"first {rows} rows, {t_one:.1f} s",
    }


def copy_reference(torch, binding):
    """Streaming reference: the library's plain copy kernel over 1 GiB (also what
    the hardware traffic counters are calibrated on).  Returns GB/s."""
    n_copy = 256 * 1024 * 1024
    src = torch.empty(n_copy, dtype=torch.float32, device="cuda:0").fill_(1.0)
    dst = torch.empty_like(src)
    binding.sgap_copy_f32(src, dst)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(10):
        binding.sgap_copy_f32(src, dst)
    torch.cuda.synchronize()
    return 2.0 * n_copy * 4 * 10 / (time.perf_counter() - t0) / 1e9


def sddmm_cpu_baseline(p, X1):
    """The SDDMM oracle on all host cores, whole workload, repeated for about 10 s."""
    import oracle

    cores = len(os.sched_getaffinity(0))
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env))
    reps, t_all = 0, 0.0
    while t_all < 10.0 and reps < 200:
        t0 = time.perf_counter()
        oracle.sddmm_csr(p.M, p.K, p.N, p.rowptr, p.colidx, p.vals, X1, p.B, nthreads=cores)
        t_all += time.perf_counter() - t0
        reps += 1
    return {
        "value": 2.0 * p.nnz * p.N * reps / t_all / 1e9,
        "unit": "GFLOP/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"whole {p.name} workload x{reps}, fp64 entry-by-entry SDDMM oracle (result and error bound), "
                  f"static row split over {cores} threads, {t_all:.1f} s",
        "seconds_per_pass": t_all / reps,
    }


def main_sddmm(a):
    """--op sddmm: the sampled dense-dense product on the workload's pattern
    (J = the workload's N, X2T = its B, X1 seeded), same JSON contract."""
    import torch

    from paper_2209_02882_amd import binding
    from paper_2209_02882_amd import workloads as wl
    from paper_2209_02882_amd.device import DeviceProblem

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.load()
    p = wl.make_problem(a.workload, N=a.ncols)
    X1h = wl.sddmm_left_operand(p)
    log(f"[bench] sddmm on {a.workload}: {p.row_stats()}")
    dp = DeviceProblem(p)
    binding.sgap_set_tuning(binding.SGAP_TUNE_LONG_ROW_MIN, a.long_row_min)
    binding.sgap_set_tuning(binding.SGAP_TUNE_PANEL_WINDOW_KB, a.window_kb)
    X1 = torch.from_numpy(X1h).cuda()
    out_vals = torch.empty(p.nnz, dtype=torch.float32, device="cuda:0")
    min_bytes = wl.sddmm_minimal_bytes(p)
    flops = 2 * p.nnz * p.N

    def run(g, st, n):
        for _ in range(n):
            dp.launch_sddmm(X1, out_vals, g, st)

    sweep = []
    if a.point:
        g, st = a.point.split(",")[:2]
        best = (int(g), st)
    else:
        for st in ("parallel", "serial"):
            for g in binding.GROUP_SIZES:
                run(g, st, 1)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                run(g, st, a.sweep_iters)
                torch.cuda.synchronize()
                t = (time.perf_counter() - t0) / a.sweep_iters
                sweep.append({"group": g, "strategy": st, "ms": t * 1e3, "gflops": flops / t / 1e9,
                              "gbs": min_bytes / t / 1e9, "hbm_frac": min_bytes / t / 1e9 / HBM_PEAK_GBS})
                log(f"[sweep] sddmm g={g:2d} {st:8s} {t * 1e3:9.3f} ms {flops / t / 1e9:9.1f} GFLOP/s "
                    f"{min_bytes / t / 1e9:8.1f} GB/s")
        b = min(sweep, key=lambda r: r["ms"])
        best = (b["group"], b["strategy"])
    g, st = best
    run(g, st, a.warmup)
    binding.sgap_profile_enable(True)
    binding.sgap_profile_collect()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(g, st, a.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_ms, n_ev = binding.sgap_profile_collect()
    binding.sgap_profile_enable(False)
    ms_per_step = elapsed / a.steps * 1e3
    kernel_avg_ms = kernel_ms / max(1, n_ev)
    achieved = min_bytes / (kernel_avg_ms * 1e-3) / 1e9
    copy_gbs = copy_reference(torch, binding)
    out = {
        "metric": "SDDMM effective GFLOP/s (2*nnz*J/t), fp32, best (group_size, strategy) point",
        "value": flops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": a.workload, "op": "sddmm", "M": p.M, "K": p.K, "J": p.N, "nnz": p.nnz,
                   "group_size": g, "strategy": st, "long_row_min": a.long_row_min},
        "copy_kernel_gbs": copy_gbs,
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_SDDMM_TRAFFIC_BYTES.get((a.workload, g, st) + ((a.long_row_min,) if a.long_row_min else ()))
            if a.ncols is None and not a.window_kb else None,
            "kernel_avg_ms": kernel_avg_ms,
            "algorithmic_bytes": min_bytes,
        },
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = sddmm_cpu_baseline(p, X1h)
    if a.sweep_out and sweep:
        with open(a.sweep_out, "w") as f:
            json.dump({"workload": a.workload, "op": "sddmm", "stats": p.row_stats(), "points": sweep}, f, indent=1)
    print(json.dumps(out), flush=True)


def main_tensor(a):
    """--op mttkrp / --op ttm: the third-order operators on a seeded random
    tensor (--workload tensor3 unless another tensor workload is named), same
    JSON contract.  TTM along the third index is SpMM over the stored fibers,
    so it sweeps all 28 SpMM points; MTTKRP sweeps (group_size, strategy)."""
    import torch

    import numpy as np

    from paper_2209_02882_amd import binding
    from paper_2209_02882_amd import workloads as wl
    from paper_2209_02882_amd.device import POINTS, DeviceTensor3

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.load()
    name = a.workload if a.workload in wl.TENSOR_WORKLOADS else "tensor3"
    p = wl.make_tensor3(name, J=a.ncols)
    log(f"[bench] {a.op} on {name}: {p.stats()}")
    dt = DeviceTensor3(p)
    ttm = a.op == "ttm"
    if ttm:
        out_t = torch.empty((p.fibers, p.J), dtype=torch.float32, device="cuda:0")
        min_bytes = p.nnz * 8 + (p.fibers + 1) * 4 + p.L * p.J * 4 + p.fibers * p.J * 4
        flops = 2 * p.nnz * p.J
        points = POINTS
        launch = lambda pt: dt.launch_ttm(out_t, *pt)
    else:
        out_t = torch.empty((p.I, p.J), dtype=torch.float32, device="cuda:0")
        min_bytes = p.mttkrp_minimal_bytes()
        flops = p.mttkrp_flops()
        points = [(g, st) for st in ("parallel", "serial") for g in binding.GROUP_SIZES]
        launch = lambda pt: dt.launch_mttkrp(out_t, *pt)

    def run(pt, n):
        for _ in range(n):
            launch(pt)

    sweep = []
    if a.point:
        f = a.point.split(",")
        best = (int(f[0]), *f[1:])
    else:
        for pt in points:
            run(pt, 1)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            run(pt, a.sweep_iters)
            torch.cuda.synchronize()
            t = (time.perf_counter() - t0) / a.sweep_iters
            sweep.append({"point": list(pt), "ms": t * 1e3, "gflops": flops / t / 1e9, "gbs": min_bytes / t / 1e9,
                          "hbm_frac": min_bytes / t / 1e9 / HBM_PEAK_GBS})
            log(f"[sweep] {a.op} {pt} {t * 1e3:9.3f} ms {flops / t / 1e9:9.1f} GFLOP/s {min_bytes / t / 1e9:8.1f} GB/s")
        best = tuple(min(sweep, key=lambda r: r["ms"])["point"])
    run(best, a.warmup)
    binding.sgap_profile_enable(True)
    binding.sgap_profile_collect()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(best, a.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_ms, n_ev = binding.sgap_profile_collect()
    binding.sgap_profile_enable(False)
    ms_per_step = elapsed / a.steps * 1e3
    kernel_avg_ms = kernel_ms / max(1, n_ev)
    achieved = min_bytes / (kernel_avg_ms * 1e-3) / 1e9
    copy_gbs = copy_reference(torch, binding)
    config = {"workload": name, "op": a.op, "I": p.I, "K": p.K, "L": p.L, "J": p.J, "fibers": p.fibers,
              "nnz": p.nnz, "group_size": best[0], "strategy": best[1]}
    if ttm:
        config["schedule"] = best[2]
    out = {
        "metric": ("TTM effective GFLOP/s (2*nnz*J/t)" if ttm else "MTTKRP effective GFLOP/s (2*(nnz+fibers)*J/t)")
                  + ", fp32, best point",
        "value": flops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": config,
        "copy_kernel_gbs": copy_gbs,
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TENSOR_TRAFFIC_BYTES.get((a.op, name, *best)) if a.ncols is None else None,
            "kernel_avg_ms": kernel_avg_ms,
            "algorithmic_bytes": min_bytes,
        },
    }
    if not a.no_cpu_baseline:
        import oracle

        cores = len(os.sched_getaffinity(0))
        env = os.environ.get("OMP_NUM_THREADS")
        if env and env.isdigit():
            cores = min(cores, int(env))
        reps, t_all = 0, 0.0
        while t_all < 10.0 and reps < 200:
            t0 = time.perf_counter()
            if ttm:
                oracle.ttm_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, p.X2, nthreads=cores)
            else:
                oracle.mttkrp_csf(p.I, p.K, p.L, p.J, p.fptr, p.fidx, p.eptr, p.eidx, p.vals, p.X1, p.X2,
                                  nthreads=cores)
            t_all += time.perf_counter() - t0
            reps += 1
        out["cpu_baseline"] = {
            "value": flops * reps / t_all / 1e9,
            "unit": "GFLOP/s",
            "cores": cores,
            "kind": "oracle",
            "sample": f"whole {name} workload x{reps}, fp64 {a.op} oracle (result and error bound), static split "
                      f"over {cores} threads, {t_all:.1f} s; rated with the same flop count as the GPU line",
            "seconds_per_pass": t_all / reps,
        }
    if a.sweep_out and sweep:
        with open(a.sweep_out, "w") as f:
            json.dump({"workload": name, "op": a.op, "stats": p.stats(), "points": sweep}, f, indent=1)
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--op", default="spmm", choices=("spmm", "sddmm", "mttkrp", "ttm"),
                    help="spmm (the headline path), sddmm on the same workload's pattern, or mttkrp / ttm on a "
                         "seeded third-order tensor")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="stencil27")
    ap.add_argument("--ncols", type=int, default=None, help="override N, the number of dense columns")
    ap.add_argument("--sweep-iters", type=int, default=3)
    ap.add_argument("--point", default=None, help="fix the point: e.g. 8,parallel,row_split (skips the sweep)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep-out", default=None, help="write the per-point sweep table (JSON) to this file")
    ap.add_argument("--long-row-min", type=int, default=0,
                    help="row-split schedule: rows of at least this many entries are produced by column windows "
                         "(SGAP_TUNE_LONG_ROW_MIN; 0 = off)")
    ap.add_argument("--window-kb", type=int, default=0, help="KiB of B per column window of that path (0 = 2048)")
    ap.add_argument("--gr", action="store_true",
                    help="also sweep the row-split points with the reduction narrower than the tiling "
                         "(group_size lanes per row, sub-groups of reduce_size < group_size merged with atomics)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build measures one GPU; run with --gpus 1 "
                 "(the path would shard by row blocks of A and C with B replicated, no exchange step)")

    if a.op == "sddmm":
        return main_sddmm(a)
    if a.op in ("mttkrp", "ttm"):
        return main_tensor(a)

    import torch

    from paper_2209_02882_amd import binding
    from paper_2209_02882_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.load()

    t0 = time.perf_counter()
    p = wl.make_problem(a.workload, N=a.ncols)
    log(f"[bench] workload {a.workload}: {p.row_stats()} generated in {time.perf_counter() - t0:.1f}s")
    log(f"[bench] recipe: {wl.recipe(a.workload)}; seed {wl.WORKLOADS[a.workload][0]}")

    from paper_2209_02882_amd.device import POINTS, DeviceProblem

    dp = DeviceProblem(p)
    C = torch.empty((p.M, p.N), dtype=torch.float32, device="cuda:0")
    binding.sgap_set_tuning(binding.SGAP_TUNE_LONG_ROW_MIN, a.long_row_min)
    binding.sgap_set_tuning(binding.SGAP_TUNE_PANEL_WINDOW_KB, a.window_kb)
    min_bytes = p.minimal_bytes()
    flops = p.flops()

    sweep = []
    if a.point:
        g, st, sc = a.point.split(",")
        best = (int(g), st, sc)
    else:
        for pt in POINTS:
            t = time_point(dp, torch, binding, C, pt, a.sweep_iters)
            sweep.append({"group": pt[0], "strategy": pt[1], "schedule": pt[2], "ms": t * 1e3,
                          "gflops": flops / t / 1e9, "gbs": min_bytes / t / 1e9,
                          "hbm_frac": min_bytes / t / 1e9 / HBM_PEAK_GBS})
            log(f"[sweep] g={pt[0]:2d} {pt[1]:8s} {pt[2]:12s} {t * 1e3:9.3f} ms "
                f"{flops / t / 1e9:9.1f} GFLOP/s {min_bytes / t / 1e9:8.1f} GB/s")
        b = min(sweep, key=lambda r: r["ms"])
        best = (b["group"], b["strategy"], b["schedule"])
    gr_sweep = []
    if a.gr:
        from paper_2209_02882_amd.device import GR_POINTS

        for g_lanes, r_lanes in GR_POINTS:
            dp.launch_gr(C, g_lanes, r_lanes)  # warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(a.sweep_iters):
                dp.launch_gr(C, g_lanes, r_lanes)
            torch.cuda.synchronize()
            t = (time.perf_counter() - t0) / a.sweep_iters
            gr_sweep.append({"group": g_lanes, "reduce": r_lanes, "ms": t * 1e3})
            log(f"[sweep] row_split parallel g={g_lanes:2d} r={r_lanes:2d} {t * 1e3:9.3f} ms")
    log(f"[bench] timing point {best}")

    g, st, sc = best
    args = (p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C, g, binding.STRATEGIES[st], binding.SCHEDULES[sc])
    for _ in range(a.warmup):
        binding.sgap_spmm_csr_ex(*args)
    binding.sgap_profile_enable(True)
    binding.sgap_profile_collect()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        binding.sgap_spmm_csr_ex(*args)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_ms, n_ev = binding.sgap_profile_collect()
    binding.sgap_profile_enable(False)
    ms_per_step = elapsed / a.steps * 1e3
    kernel_avg_ms = kernel_ms / max(1, n_ev)

    copy_gbs = copy_reference(torch, binding)

    # per-launch figures outside the timed region: median and minimum of 25
    # launches, warm and with every cache overwritten before each launch
    warm = launch_stats(torch, lambda: binding.sgap_spmm_csr_ex(*args), 25)
    flush = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")  # 1 GiB
    cold = launch_stats(torch, lambda: binding.sgap_spmm_csr_ex(*args), 25, flush=flush)
    del flush

    achieved = min_bytes / (kernel_avg_ms * 1e-3) / 1e9
    out = {
        "metric": "SpMM effective GFLOP/s (2*nnz*N/t), fp32, best (group_size, strategy, schedule) point",
        "value": flops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": a.workload, "M": p.M, "K": p.K, "N": p.N, "nnz": p.nnz,
                   "group_size": g, "strategy": st, "schedule": sc, "long_row_min": a.long_row_min},
        "hbm_gbs_minimal_bytes": min_bytes / (ms_per_step * 1e-3) / 1e9,
        "hbm_frac_minimal_bytes": min_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "copy_kernel_gbs": copy_gbs,
        "launch_ms_warm": warm,
        "launch_ms_caches_flushed": cold,
        "ceilings": ceilings(p),
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get((a.workload, g, st, sc) + ((a.long_row_min,) if a.long_row_min else ()))
            if a.ncols is None and not a.window_kb else None,
            "kernel_avg_ms": kernel_avg_ms,
            "algorithmic_bytes": min_bytes,
        },
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(p)
    if a.sweep_out and sweep:
        with open(a.sweep_out, "w") as f:
            json.dump({"workload": a.workload, "stats": p.row_stats(), "points": sweep, "gr_points": gr_sweep}, f,
                      indent=1)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
