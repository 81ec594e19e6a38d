#!/usr/bin/env python3
"""Benchmark of the CSR SpMM hot path on one MI355X.

A "step" is one whole SpMM call (everything the call enqueues: row zeroing,
the preparation of the window path, the kernels) on a seeded synthetic
workload that is resident in HBM.  For each of the three large workloads
(stencil27, rmat, skewed) every selectable path is swept briefly: the 28
(group_size, strategy, schedule) points and the row-split points with their
long rows taken by column windows; the best one is then timed for exactly
--steps steps.  ONE JSON line goes to stdout: its top-level fields are the
headline workload's (--workload, default skewed, the largest), `per_workload`
carries all three, each with its HBM roofline (minimal bytes
nnz*8 + (M+1)*4 + K*N*4 + M*N*4 over the event-timed duration of the whole
call) and the CPU oracle timed on the host next to it.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2209_02882_amd.profile_summary import kernel_source_hash  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth
FP32_VECTOR_PEAK_TFLOPS = 157.3  # MI355X published fp32 vector rate
# Rate at which 256 compute units deliver gathered dwordx4 operands that hit in
# L1, measured with paper_2209_02882_amd/microbench/gather_bandwidth.hip
# (profiles/microbenchmarks.md): 55-60 bytes per clock per compute unit.
L1_GATHER_TBS = 36.0
LARGE_WORKLOADS = ("stencil27", "rmat", "skewed")


def measured_traffic(op: str, workload: str, config: dict):
    """HBM bytes per call from a committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE scaled by the same counters on a plain copy): the profiles/*.md that
    holds a `traffic-record:` line for this operator, workload and configuration.
    Returns (bytes, file) when the record was taken at the kernel sources as they
    are now, else (None, reason): a figure from other sources says nothing about
    these kernels."""
    now = kernel_source_hash()
    stale = None
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        for line in open(path):
            if not line.startswith("traffic-record:"):
                continue
            rec = json.loads(line[len("traffic-record:"):])
            if rec.get("op") != op or rec.get("workload") != workload or rec.get("config") != config:
                continue
            if rec.get("source_sha256") == now:
                return int(rec["bytes"]), os.path.relpath(path, ROOT)
            stale = os.path.relpath(path, ROOT)
    return None, (f"{stale} was taken at other kernel sources" if stale else "no profile of this configuration")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_config(dp, torch, C, cfg, ws, iters):
    """Seconds per call of one configuration: a warm-up, then `iters` calls between synchronisations."""
    dp.launch_cfg(C, cfg, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        dp.launch_cfg(C, cfg, ws)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / iters


def describe(cfg, binding) -> dict:
    """The fields of a configuration that name the path: the point, and every knob that is not left to the library."""
    d = {"group_size": cfg.group_size, "strategy": binding.STRATEGY_NAMES[cfg.strategy],
         "schedule": binding.SCHEDULE_NAMES[cfg.schedule]}
    for k, v in cfg.as_dict().items():
        if k not in ("group_size", "strategy", "schedule") and v != (-1 if k == "xcd_remap" else 0):
            d[k] = v
    return d


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


def cpu_baseline(p, seconds=10.0):
    """The oracle as it stands, timed on this host: all cores on the whole
    workload (static row split) repeated for about `seconds`, and one core on the
    first quarter of the rows."""
    import oracle

    cores = len(os.sched_getaffinity(0))
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        cores = min(cores, int(env))
    # all cores: the whole workload, repeated until about 10 s of wall time
    reps, t_all = 0, 0.0
    while t_all < seconds and reps < 200:
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
    """Streaming references over 1 GiB: the library's copy, read-only and write-only kernels (the copy is also
    what the hardware traffic counters are calibrated on).  Returns GB/s of each, bytes moved over time."""
    n = 256 * 1024 * 1024
    src = torch.empty(n, dtype=torch.float32, device="cuda:0").fill_(1.0)
    dst = torch.empty_like(src)
    sink = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    out = {}
    for name, mode, s_, d_, moved in (("copy", 0, src, dst, 2 * n * 4), ("read", 1, src, sink, n * 4),
                                      ("write", 2, None, dst, n * 4)):
        binding.sgap_stream_f32(s_, d_, n, mode)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(10):
            binding.sgap_stream_f32(s_, d_, n, mode)
        torch.cuda.synchronize()
        out[name] = moved * 10 / (time.perf_counter() - t0) / 1e9
    return out


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
    X1 = torch.from_numpy(X1h).cuda()
    out_vals = torch.empty(p.nnz, dtype=torch.float32, device="cuda:0")
    min_bytes = wl.sddmm_minimal_bytes(p)
    flops = 2 * p.nnz * p.N
    ws_size = binding.sgap_sddmm_csr_workspace_size(p.K, p.N, a.window_kb) if a.long_row_min else 0
    ws = torch.empty(ws_size, dtype=torch.uint8, device="cuda:0") if ws_size else None

    def run(g, st, n):
        for _ in range(n):
            if a.long_row_min:
                binding.sgap_sddmm_csr_windows(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, X1, dp.B, out_vals, g,
                                               binding.STRATEGIES[st], a.long_row_min, a.window_kb, workspace=ws)
            else:
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
    key = {"group_size": g, "strategy": st}
    if a.long_row_min:
        key["long_row_min"] = a.long_row_min
    traffic, traffic_from = (None, "J or the window was overridden") if a.ncols or a.window_kb else \
        measured_traffic("sddmm", a.workload, key)
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
        "stream_kernels_gbs": copy_gbs,
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_from": traffic_from,
            "call_avg_ms": kernel_avg_ms,
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
    so it sweeps all 28 SpMM points; MTTKRP sweeps its 28 (group_size, strategy,
    schedule) points: slices or stored entries as the unit of work."""
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
        points = [(g, st, sc) for sc in ("row_split", "nnz_balanced") for st in ("parallel", "serial")
                  for g in binding.GROUP_SIZES]
        launch = lambda pt: dt.launch_mttkrp(out_t, *(pt if len(pt) == 3 else (*pt, "row_split")))

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
    if len(best) == 2:
        best = (*best, "row_split")
    key = {"group_size": best[0], "strategy": best[1], "schedule": best[2]}
    traffic, traffic_from = (None, "J was overridden") if a.ncols else measured_traffic(a.op, name, key)
    config = {"workload": name, "op": a.op, "I": p.I, "K": p.K, "L": p.L, "J": p.J, "fibers": p.fibers,
              "nnz": p.nnz, "group_size": best[0], "strategy": best[1], "schedule": best[2]}
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
        "stream_kernels_gbs": copy_gbs,
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_from": traffic_from,
            "call_avg_ms": kernel_avg_ms,
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


def candidates(p, binding, with_gr):
    """Every selectable path: the 28 points; the row-split points with their long rows by column windows
    (where the operands allow 16-byte loads and the matrix has rows that long); optionally the 21 points
    with the reduction narrower than the tiling."""
    import numpy as np

    from paper_2209_02882_amd.device import GR_POINTS, POINTS

    out = [binding.make_config(*pt) for pt in POINTS]
    longest = int(np.diff(p.rowptr.astype(np.int64)).max()) if p.M else 0
    if p.N % 4 == 0:
        for min_len in (1024, 4096):
            if longest < min_len:
                continue
            for st, groups in (("serial", (1, 2, 4, 8)), ("parallel", (1, 4, 8))):
                out += [binding.make_config(g, st, "row_split", long_row_min=min_len) for g in groups]
    if with_gr:
        out += [binding.make_config(g, "parallel", "row_split", reduce_size=r) for g, r in GR_POINTS]
    return out


def reordered_rows(dp, torch, binding, C, cfg, ws, cfg_d):
    """The same configuration on the copies of the matrix that sgap_reorder_rows_csr writes (rows grouped by
    first column, by length): time of the pass and of a call on the copy, whose product has its rows in the
    new order.  An option a caller has, not part of the headline."""
    import copy

    p = dp.p
    dev = dp.rowptr.device
    perm = torch.empty(p.M, dtype=torch.int32, device=dev)
    rowptr = torch.empty_like(dp.rowptr)
    colidx = torch.empty_like(dp.colidx)
    vals = torch.empty_like(dp.vals)
    order_ws = torch.empty(binding.sgap_reorder_rows_workspace_size(p.M), dtype=torch.uint8, device=dev)
    out = []
    for order in ("first_column", "length"):
        run = lambda: binding.sgap_reorder_rows_csr(p.M, p.K, dp.rowptr, dp.colidx, dp.vals, order, perm, rowptr,
                                                    colidx, vals, order_ws)
        pre = launch_stats(torch, run, 5)
        dq = copy.copy(dp)
        dq.rowptr, dq.colidx, dq.vals = rowptr, colidx, vals
        # the configuration that won on the stored order, and the nnz-balanced serial points with more entries
        # per lane (rows of one length now lie together)
        best_t, best_c = time_config(dq, torch, C, cfg, ws, 20), cfg_d
        for g in (16, 32, 64):
            other = binding.make_config(g, "serial", "nnz_balanced")
            if describe(other, binding) == cfg_d:
                continue
            t = time_config(dq, torch, C, other, None, 20)
            if t < best_t:
                best_t, best_c = t, describe(other, binding)
        out.append({"order": order, "preprocessing_ms": pre["median"], "ms_per_step": best_t * 1e3, "config": best_c})
        log(f"[bench] {p.name}: rows by {order}: pass {pre['median']:.3f} ms, call {best_t * 1e3:.3f} ms with {best_c}")
    return out


def measure_spmm(a, name, torch, binding, wl, copy_gbs):
    """Sweep, time and rate one workload; returns its record of the JSON line."""
    from paper_2209_02882_amd.device import DeviceProblem

    t0 = time.perf_counter()
    p = wl.make_problem(name, N=a.ncols)
    log(f"[bench] workload {name}: {p.row_stats()} generated in {time.perf_counter() - t0:.1f}s")
    log(f"[bench] recipe: {wl.recipe(name)}; seed {wl.WORKLOADS[name][0]}")
    dp = DeviceProblem(p, arena=not a.separate_allocations)
    C = dp.new_output()
    min_bytes = p.minimal_bytes()
    flops = p.flops()
    if a.reorder:
        # everything below runs on the copy that sgap_reorder_rows_csr writes (rows of C come out in its order)
        perm = torch.empty(p.M, dtype=torch.int32, device="cuda:0")
        new = [torch.empty_like(t) for t in (dp.rowptr, dp.colidx, dp.vals)]
        order_ws = torch.empty(binding.sgap_reorder_rows_workspace_size(p.M), dtype=torch.uint8, device="cuda:0")
        binding.sgap_reorder_rows_csr(p.M, p.K, dp.rowptr, dp.colidx, dp.vals, a.reorder, perm, *new, order_ws)
        torch.cuda.synchronize()
        dp.rowptr, dp.colidx, dp.vals = new
        del order_ws, perm

    sweep = []
    if a.point:
        f = a.point.split(",")
        knobs = dict(kv.split("=") for kv in f[3:])
        best = binding.make_config(int(f[0]), f[1], f[2], **{k: int(v) for k, v in knobs.items()})
    else:
        best, best_t = None, None
        for cfg in candidates(p, binding, a.gr):
            ws = dp.workspace_for(cfg)
            t = time_config(dp, torch, C, cfg, ws, a.sweep_iters)
            d = describe(cfg, binding)
            sweep.append({**d, "ms": t * 1e3, "gflops": flops / t / 1e9, "gbs": min_bytes / t / 1e9,
                          "hbm_frac": min_bytes / t / 1e9 / HBM_PEAK_GBS})
            log(f"[sweep] {name} {d} {t * 1e3:9.3f} ms {flops / t / 1e9:9.1f} GFLOP/s {min_bytes / t / 1e9:8.1f} GB/s")
            if best_t is None or t < best_t:
                best, best_t = cfg, t
            del ws
    ws = dp.workspace_for(best)
    best_d = describe(best, binding)
    if a.reorder:
        best_d["row_order"] = a.reorder
    log(f"[bench] {name}: timing {best_d}")

    for _ in range(a.warmup):
        dp.launch_cfg(C, best, ws)
    binding.sgap_profile_enable(True)
    binding.sgap_profile_collect()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        dp.launch_cfg(C, best, ws)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    call_ms, n_ev = binding.sgap_profile_collect()
    binding.sgap_profile_enable(False)
    ms_per_step = elapsed / a.steps * 1e3
    call_avg_ms = call_ms / max(1, n_ev)  # all kernels of a call, between events on the launch stream

    # per-launch figures outside the timed region: median and minimum of 25
    # launches, warm and with every cache overwritten before each launch
    warm = launch_stats(torch, lambda: dp.launch_cfg(C, best, ws), 25)
    flush = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")  # 1 GiB
    cold = launch_stats(torch, lambda: dp.launch_cfg(C, best, ws), 25, flush=flush)
    del flush

    achieved = min_bytes / (call_avg_ms * 1e-3) / 1e9
    traffic, traffic_from = (None, "N or the point was overridden") if a.ncols else measured_traffic("spmm", name, best_d)
    rec = {
        "value": flops / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "ms_per_step": ms_per_step,
        "config": {"workload": name, "M": p.M, "K": p.K, "N": p.N, "nnz": p.nnz, **best_d},
        "hbm_gbs_minimal_bytes": min_bytes / (ms_per_step * 1e-3) / 1e9,
        "hbm_frac_minimal_bytes": min_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "launch_ms_warm": warm,
        "launch_ms_caches_flushed": cold,
        "ceilings": ceilings(p),
        "device_memory": ("one allocation per operand" if a.separate_allocations else
                          "rowptr, colidx, vals, B and C packed into one allocation at 512-byte boundaries"),
        "roofline": {
            "bound": "hbm",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_from": traffic_from,
            "call_avg_ms": call_avg_ms,
            "includes": "every kernel the call enqueues (row zeroing, window preparation)",
            "algorithmic_bytes": min_bytes,
        },
    }
    if not a.no_reorder and not a.point and not a.reorder:
        rec["reordered_rows"] = reordered_rows(dp, torch, binding, C, best, ws, best_d)
    if not a.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(p, a.cpu_seconds)
    if a.sweep_out and sweep:
        with open(a.sweep_out.replace("{workload}", name), "w") as fh:
            json.dump({"workload": name, "stats": p.row_stats(), "points": sweep}, fh, indent=1)
    if a.tuner_out:
        # the library's own tuner (sgap_autotune_csr_cfg) over the space it has, with the working memory the
        # window configurations at their defaults need
        tune_ws = dp.workspace_for(binding.make_config(1, "serial", "row_split", long_row_min=1024))
        t0 = time.perf_counter()
        t_best, table = binding.sgap_autotune_csr_cfg(p.M, p.K, p.N, dp.rowptr, dp.colidx, dp.vals, dp.B, C,
                                                      workspace=tune_ws)
        log(f"[bench] {name}: tuner rated {len(table)} configurations in {time.perf_counter() - t0:.1f} s; "
            f"best {describe(t_best.config, binding)} {t_best.ms:.3f} ms")
        with open(a.tuner_out.replace("{workload}", name), "w") as fh:
            json.dump({"workload": name, "stats": p.row_stats(),
                       "best": {**describe(t_best.config, binding), "ms": t_best.ms},
                       "table": [{**describe(t.config, binding), "ms": t.ms} for t in table]}, fh, indent=1)
        del tune_ws
    del dp, C, ws
    # (no torch.cuda.empty_cache() here: device memory that was freed and allocated again serves random
    # gathers measurably slower on this machine, rmat on the reordered copy 0.71 -> 0.87 ms; the next workload
    # takes its tensors out of the blocks torch keeps)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--op", default="spmm", choices=("spmm", "sddmm", "mttkrp", "ttm"),
                    help="spmm (the headline path), sddmm on the same workload's pattern, or mttkrp / ttm on a "
                         "seeded third-order tensor")
    ap.add_argument("--tuner-out", default=None,
                    help="spmm: also run the library's tuner and write its table here as JSON ({workload} is replaced)")
    ap.add_argument("--reorder", default=None, choices=("first_column", "length"),
                    help="spmm: run on the copy of the matrix that sgap_reorder_rows_csr writes with this key")
    ap.add_argument("--separate-allocations", action="store_true",
                    help="spmm: one device allocation per operand instead of all five arrays packed into one "
                         "(results are the same; kernels that gather at random are slower: R-MAT 0.86 against 0.70 ms)")
    ap.add_argument("--no-reorder", action="store_true",
                    help="skip the leg that times the best configuration on the reordered copies of the matrix")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None,
                    help="the workload of the line's top-level fields (spmm: skewed, the largest configuration)")
    ap.add_argument("--others", default=None,
                    help="spmm: further workloads to carry in per_workload, comma separated (default: the other large "
                         "configurations; '' for none)")
    ap.add_argument("--ncols", type=int, default=None, help="override N, the number of dense columns")
    ap.add_argument("--sweep-iters", type=int, default=3)
    ap.add_argument("--point", default=None,
                    help="fix the point: e.g. 8,parallel,row_split or 4,serial,row_split,long_row_min=1024 "
                         "(skips the sweep)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=8.0, help="wall time of the oracle's all-core leg per workload")
    ap.add_argument("--sweep-out", default=None,
                    help="write the per-point sweep table (JSON) to this file ({workload} in the name is replaced)")
    ap.add_argument("--long-row-min", type=int, default=0,
                    help="sddmm: entries of rows of at least this many entries are produced by column windows (0 = off)")
    ap.add_argument("--window-kb", type=int, default=0, help="sddmm: KiB of X2T per column window of that path (0 = 2048)")
    ap.add_argument("--gr", action="store_true",
                    help="also sweep the row-split points with the reduction narrower than the tiling "
                         "(group_size lanes per row, sub-groups of reduce_size < group_size merged with atomics)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build measures one GPU; run with --gpus 1 "
                 "(the path would shard by row blocks of A and C with B replicated, no exchange step)")

    if a.op == "sddmm":
        a.workload = a.workload or "stencil27"
        return main_sddmm(a)
    if a.op in ("mttkrp", "ttm"):
        a.workload = a.workload or "tensor3"
        return main_tensor(a)

    import torch

    from paper_2209_02882_amd import binding
    from paper_2209_02882_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    binding.load()
    headline = a.workload or "skewed"
    if a.others is None:
        others = [w for w in LARGE_WORKLOADS if w != headline] if a.workload is None and not a.point else []
    else:
        others = [w for w in a.others.split(",") if w]
    copy_gbs = copy_reference(torch, binding)

    per_workload = {}
    for name in [headline] + others:  # the headline in the fresh process
        per_workload[name] = measure_spmm(a, name, torch, binding, wl, copy_gbs)
    h = per_workload[headline]
    out = {
        "metric": "SpMM effective GFLOP/s (2*nnz*N/t), fp32, best (group_size, strategy, schedule) point",
        "value": h["value"],
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": h["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": h["config"],
        "hbm_gbs_minimal_bytes": h["hbm_gbs_minimal_bytes"],
        "hbm_frac_minimal_bytes": h["hbm_frac_minimal_bytes"],
        "stream_kernels_gbs": copy_gbs,
        "launch_ms_warm": h["launch_ms_warm"],
        "launch_ms_caches_flushed": h["launch_ms_caches_flushed"],
        "ceilings": h["ceilings"],
        "roofline": h["roofline"],
        "kernel_source_sha256": kernel_source_hash(),
    }
    if "cpu_baseline" in h:
        out["cpu_baseline"] = h["cpu_baseline"]
    out["per_workload"] = per_workload
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
