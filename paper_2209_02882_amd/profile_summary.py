"""Turn the output of a set of rocprofv3 runs of bench.py into the short
summary that is kept under profiles/: per-kernel durations (--kernel-trace
--stats), hardware counters per dispatch (--pmc passes), HBM bytes per call
calibrated on the library's copy kernel, and a machine-readable
`traffic-record:` line that bench.py reads back for roofline.traffic.

    python -m paper_2209_02882_amd.profile_summary RUN_DIR --title "..." \
        --op spmm --workload skewed --config '{"group_size": 1, ...}' --out profiles/NAME.md

RUN_DIR holds one sub-directory per rocprofv3 run (any names), each with the
CSV files rocprofv3 wrote (`*_kernel_stats.csv`, `*_counter_collection.csv`)
and, optionally, `command.txt` (the full command of the run) and `bench.json`
(the line bench.py printed).  Nothing here runs on the GPU.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KERNEL = "copy_f32_kernel"
COPY_KIB = 1024 * 1024.0  # the copy moves 1 GiB in and 1 GiB out per dispatch
NOT_THE_CALL = (COPY_KERNEL, "read_f32_kernel", "write_f32_kernel", "at::native", "elementwise")


def kernel_source_hash() -> str:
    """sha256 over the kernel sources (csrc/*.hip, *.hpp, sorted by name): what a
    measured traffic figure is tied to."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2209_02882_amd", "csrc")
    for name in sorted(os.listdir(src)):
        if name.endswith((".hip", ".hpp")):
            h.update(name.encode())
            h.update(open(os.path.join(src, name), "rb").read())
    return h.hexdigest()


def short(name: str) -> str:
    name = name.split("(")[0]
    return name.replace("void ", "").replace("sgap::", "")


def read_run_dir(run_dir):
    stats, counters, commands, bench = {}, collections.defaultdict(list), [], None
    for sub in sorted(os.listdir(run_dir)):
        d = os.path.join(run_dir, sub)
        if not os.path.isdir(d):
            continue
        cmd = os.path.join(d, "command.txt")
        if os.path.exists(cmd):
            commands.append(open(cmd).read().strip())
        bj = os.path.join(d, "bench.json")
        if os.path.exists(bj) and bench is None:
            try:
                bench = json.loads(open(bj).read().strip().splitlines()[-1])
            except (ValueError, IndexError):
                pass
        for f in glob.glob(os.path.join(d, "**", "*_kernel_stats.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                stats[short(r["Name"])] = r
        for f in glob.glob(os.path.join(d, "**", "*_counter_collection.csv"), recursive=True):
            for r in csv.DictReader(open(f)):
                counters[(short(r["Kernel_Name"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    return stats, counters, commands, bench


SHAPE_KEYS = ("workload", "op", "M", "K", "N", "nnz", "J", "I", "L", "fibers", "rank")  # what bench.py adds to a configuration's description


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("run_dir")
    ap.add_argument("--title", required=True)
    ap.add_argument("--op", default=None, help="default: the one the run's bench.py line names, else spmm")
    ap.add_argument("--workload", default=None, help="default: the one the run's bench.py line names")
    ap.add_argument("--config", default=None,
                    help="JSON: the configuration as bench.py describes it (default: the one of the run's bench.py line)")
    ap.add_argument("--out", required=True)
    ap.add_argument("--note", default="")
    ap.add_argument("--also", action="append", default=[], metavar="RUN_DIR::CONFIG_JSON",
                    help="a further run directory (FETCH_SIZE and WRITE_SIZE passes are enough) whose traffic record "
                         "for another configuration of the same workload is appended")
    a = ap.parse_args()
    stats, counters, commands, bench = read_run_dir(a.run_dir)
    named = dict(bench.get("config", {})) if bench else {}
    if a.workload is None:
        a.workload = named.get("workload")
    if a.op is None:
        a.op = named.get("op", "spmm")
    if named.get("long_row_min") == 0:
        del named["long_row_min"]
    for shape in SHAPE_KEYS:
        named.pop(shape, None)
    config = json.loads(a.config) if a.config else named
    if not a.workload or not config:
        ap.error("the run holds no bench.py line: give --workload and --config")

    lines = [f"# {a.title}", ""]
    if a.note:
        lines += [a.note, ""]
    lines += ["Commands (one MI355X; run from the repository root after `cd /tmp && export TMPDIR=/tmp`, paths made absolute):",
              "", "```"] + commands + ["```", ""]
    if bench:
        keep = {k: bench[k] for k in ("value", "unit", "ms_per_step", "config") if k in bench}
        if "roofline" in bench:
            keep["roofline"] = {k: v for k, v in bench["roofline"].items() if k in ("achieved", "frac", "call_avg_ms", "algorithmic_bytes")}
        lines += ["bench.py line of the kernel-trace run (profiler attached):", "", "```", json.dumps(keep), "```", ""]

    ours = [k for k in stats if not any(s in k for s in NOT_THE_CALL)]
    if stats:
        lines += ["## rocprofv3 --kernel-trace --stats", "", "| kernel | calls | avg ns | min ns | max ns |", "|---|---|---|---|---|"]
        for k in sorted(stats, key=lambda k: -float(stats[k]["TotalDurationNs"])):
            r = stats[k]
            if k in ours or COPY_KERNEL in k:
                lines.append(f"| `{k[:100]}` | {r['Calls']} | {float(r['AverageNs']):.0f} | {r['MinNs']} | {r['MaxNs']} |")
        calls = max((int(stats[k]["Calls"]) for k in ours), default=0)
        total = sum(float(stats[k]["TotalDurationNs"]) for k in ours)
        if calls:
            lines += ["", f"All kernels of one call: {total / calls / 1e6:.3f} ms (sum of the averages over {calls} calls)."]
        lines.append("")

    names = sorted({c for _, c in counters})
    kernels = sorted({k for k, _ in counters if not any(s in k for s in NOT_THE_CALL[1:])})
    if names:
        # counters down, kernels across (those that take at least 1 % of the call's time, and the copy kernel)
        total_ns = sum(float(stats[k]["TotalDurationNs"]) for k in ours) if stats else 0.0
        shown = [k for k in kernels if COPY_KERNEL in k or not stats or k not in stats
                 or float(stats[k]["TotalDurationNs"]) >= 0.01 * total_ns]
        lines += ["## rocprofv3 --pmc (mean per dispatch)", "", "| counter | " + " | ".join(f"`{k[:44]}`" for k in shown) + " |",
                  "|---|" + "---|" * len(shown)]
        for c in names:
            row = []
            for k in shown:
                v = counters.get((k, c))
                row.append(f"{sum(v) / len(v):,.0f}" if v else "")
            lines.append(f"| {c} | " + " | ".join(row) + " |")
        lines.append("")
        derived = []
        for k in shown:
            get = lambda c: (sum(counters[(k, c)]) / len(counters[(k, c)])) if counters.get((k, c)) else None
            hit, miss = get("TCC_HIT_sum"), get("TCC_MISS_sum")
            busy, active = get("TA_BUSY_avr"), get("GRBM_GUI_ACTIVE")
            conf, lds = get("SQ_LDS_BANK_CONFLICT"), get("SQ_LDS_IDX_ACTIVE")
            parts = []
            if hit is not None and miss is not None and hit + miss > 0:
                parts.append(f"L2 hit rate {100 * hit / (hit + miss):.1f} %")
            if busy is not None and active:
                # GRBM_GUI_ACTIVE adds up the 8 dies' clocks; TA_BUSY counts clocks of one address unit
                clocks = active / 8.0
                parts.append(f"address units busy {100 * busy / clocks:.0f} % of the kernel's clocks on average"
                             + (f", {100 * get('TA_BUSY_max') / clocks:.0f} % on the busiest" if get("TA_BUSY_max") else ""))
            if conf is not None and lds:
                parts.append(f"LDS bank conflicts {100 * conf / lds:.1f} % of the LDS's active cycles")
            elif conf is not None:
                parts.append(f"LDS bank conflict cycles {conf:,.0f}")
            if get("TCC_ATOMIC_sum") is not None:
                parts.append(f"atomic requests at L2 {get('TCC_ATOMIC_sum'):,.0f}")
            if get("SQ_INSTS_VALU") is not None and get("SQ_INSTS_SALU") is not None and get("SQ_WAVES"):
                parts.append(f"per wavefront {get('SQ_INSTS_VALU') / get('SQ_WAVES'):,.0f} vector and "
                             f"{get('SQ_INSTS_SALU') / get('SQ_WAVES'):,.0f} scalar instructions")
            if parts:
                derived.append(f"- `{k[:60]}`: " + "; ".join(parts) + ".")
        if derived:
            lines += ["Derived:", ""] + derived + [""]

    extra_records = []
    for spec in a.also:
        other_dir, other_cfg = spec.split("::", 1)
        _, oc, ocmds, _ = read_run_dir(other_dir)
        ok = sorted({k for k, _ in oc if not any(s_ in k for s_ in NOT_THE_CALL[1:])})
        cp = [k for k in ok if COPY_KERNEL in k]
        if not cp or not oc.get((cp[0], "FETCH_SIZE")) or not oc.get((cp[0], "WRITE_SIZE")):
            raise SystemExit(f"{other_dir}: no calibrated FETCH_SIZE / WRITE_SIZE passes")
        fs = COPY_KIB / (sum(oc[(cp[0], "FETCH_SIZE")]) / len(oc[(cp[0], "FETCH_SIZE")]))
        ws = COPY_KIB / (sum(oc[(cp[0], "WRITE_SIZE")]) / len(oc[(cp[0], "WRITE_SIZE")]))
        mine_o = [k for k in ok if COPY_KERNEL not in k]
        calls_o = max((len(oc.get((k, "FETCH_SIZE"), [])) for k in mine_o), default=0)
        tot = sum((sum(oc.get((k, "FETCH_SIZE"), [])) * fs + sum(oc.get((k, "WRITE_SIZE"), [])) * ws) * 1024 for k in mine_o)
        extra_records.append((json.loads(other_cfg), int(round(tot / calls_o)) if calls_o else 0, ocmds))

    # HBM bytes per call from FETCH_SIZE / WRITE_SIZE, calibrated on the copy kernel (1 GiB in, 1 GiB out)
    record = None
    copy = [k for k in kernels if COPY_KERNEL in k]
    if copy and counters.get((copy[0], "FETCH_SIZE")) and counters.get((copy[0], "WRITE_SIZE")):
        f_scale = COPY_KIB / (sum(counters[(copy[0], "FETCH_SIZE")]) / len(counters[(copy[0], "FETCH_SIZE")]))
        w_scale = COPY_KIB / (sum(counters[(copy[0], "WRITE_SIZE")]) / len(counters[(copy[0], "WRITE_SIZE")]))
        lines += [f"Calibration: the copy kernel moves 1,048,576 KiB in and out per dispatch; it reads FETCH_SIZE x {f_scale:.3f} "
                  f"and WRITE_SIZE x {w_scale:.3f} KiB.", "", "| kernel | dispatches | HBM read bytes | HBM write bytes |", "|---|---|---|---|"]
        mine = [k for k in kernels if COPY_KERNEL not in k]
        calls = max((len(counters.get((k, "FETCH_SIZE"), [])) for k in mine), default=0)
        total = 0.0
        for k in mine:
            f, w = counters.get((k, "FETCH_SIZE"), []), counters.get((k, "WRITE_SIZE"), [])
            fb = sum(f) * f_scale * 1024 / calls if calls else 0.0
            wb = sum(w) * w_scale * 1024 / calls if calls else 0.0
            total += fb + wb
            lines.append(f"| `{k[:80]}` | {len(f)} | {fb:,.0f} | {wb:,.0f} |")
        lines += ["", f"HBM bytes per call (all kernels of the call, {calls} calls): {total:,.0f}"]
        if bench and "roofline" in bench:
            alg = bench["roofline"]["algorithmic_bytes"]
            lines.append(f"Algorithmic bytes per call: {alg:,} ({total / alg:.2f}x)")
        lines.append("")
        record = {"op": a.op, "workload": a.workload, "config": config, "bytes": int(round(total)),
                  "source_sha256": kernel_source_hash()}
    if record:
        lines += ["Read back by bench.py (roofline.traffic) while the kernel sources are the ones this was taken at:", "",
                  "traffic-record: " + json.dumps(record), ""]
    for cfg, nbytes, ocmds in extra_records:
        lines += [f"The same two counters for the configuration {json.dumps(cfg)} (commands as above with its --point): "
                  f"{nbytes:,} bytes per call.", "",
                  "traffic-record: " + json.dumps({"op": a.op, "workload": a.workload, "config": cfg, "bytes": nbytes,
                                                   "source_sha256": kernel_source_hash()}), ""]
    with open(a.out, "w") as fh:
        fh.write("\n".join(lines))
    print("wrote", a.out)


if __name__ == "__main__":
    main()
