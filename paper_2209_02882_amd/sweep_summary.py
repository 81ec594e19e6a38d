"""Markdown tables out of the JSON files that bench.py writes with --sweep-out and --tuner-out.

    python -m paper_2209_02882_amd.sweep_summary spmm  --dir OUT_DIR --out profiles/sweep_all_points.md W1 W2 ...
    python -m paper_2209_02882_amd.sweep_summary tuner --dir OUT_DIR --out profiles/tuner_table.md W1 W2 ...
    python -m paper_2209_02882_amd.sweep_summary other --dir OUT_DIR --out profiles/sweep_sddmm.md sddmm_W1 sddmm_W2 ...

`spmm` reads sweep_W.json (every point bench.py timed: the 28 (group size, strategy, schedule) points, the
row-split points with long rows by column windows, with --gr the points whose reduction is narrower than
their tiling); `tuner` reads tuner_W.json (the table sgap_autotune_csr_cfg filled) and compares the best
fixed configuration with the choice per workload, the comparison of the paper's Table 5.  Formatting only:
every number is one that bench.py measured and wrote.
"""
from __future__ import annotations

import argparse
import json
import math
import os

G = (1, 2, 4, 8, 16, 32, 64)
POINT_KEYS = ("group_size", "strategy", "schedule")


def name_of(d: dict) -> str:
    extra = ", ".join(f"{k}={v}" for k, v in d.items() if k not in POINT_KEYS and k not in ("ms", "gflops", "gbs", "hbm_frac"))
    return f"G={d['group_size']} {d['strategy']} {d['schedule']}" + (f" ({extra})" if extra else "")


def plain(d: dict) -> bool:
    return all(k in POINT_KEYS or k in ("ms", "gflops", "gbs", "hbm_frac") for k in d)


def header(d: dict) -> str:
    st = d["stats"]
    return (f"## {d['workload']}  (M={st['M']:,} N={st['N']} nnz={st['nnz']:,} max row {st['max_row']:,} "
            f"empty rows {st['empty_rows']:,})")


def spmm_tables(d: dict) -> list[str]:
    pts = d["points"]
    best = min(pts, key=lambda r: r["ms"])
    out = [header(d), "", "| schedule | strategy | " + " | ".join(f"G={g}" for g in G) + " |", "|---|---|" + "---|" * len(G)]
    for sc in ("row_split", "nnz_balanced"):
        for stg in ("parallel", "serial"):
            cells = []
            for g in G:
                r = [x for x in pts if plain(x) and (x["group_size"], x["strategy"], x["schedule"]) == (g, stg, sc)]
                cells.append("" if not r else (f"**{r[0]['ms']:.3f}**" if r[0] is best else f"{r[0]['ms']:.3f}"))
            out.append(f"| {sc} | {stg} | " + " | ".join(cells) + " |")
    out.append("")
    windows = [x for x in pts if "long_row_min" in x]
    if windows:
        out += ["Row-split points with the rows of at least `long_row_min` entries taken by column windows:", "",
                "| strategy | long_row_min | " + " | ".join(f"G={g}" for g in G[:4]) + " |", "|---|---|" + "---|" * 4]
        for stg in ("serial", "parallel"):
            for m in sorted({x["long_row_min"] for x in windows}):
                cells = []
                for g in G[:4]:
                    r = [x for x in windows if (x["group_size"], x["strategy"], x["long_row_min"]) == (g, stg, m)]
                    cells.append("" if not r else (f"**{r[0]['ms']:.3f}**" if r[0] is best else f"{r[0]['ms']:.3f}"))
                out.append(f"| {stg} | {m} | " + " | ".join(cells) + " |")
        out.append("")
    gr = [x for x in pts if "reduce_size" in x]
    if gr:
        out += ["Table 1's experiment: g lanes per row, reduction width r <= g (r < g merges the g/r sub-group sums of a "
                "row with atomics; r = g is the row-split parallel point above):", "",
                "| lanes per row g | " + " | ".join(f"r={r}" for r in G) + " |", "|---|" + "---|" * len(G)]
        for g in G[1:]:
            cells = []
            for r in G:
                if r > g:
                    cells.append("")
                elif r == g:
                    x = [x for x in pts if plain(x) and (x["group_size"], x["strategy"], x["schedule"]) == (g, "parallel", "row_split")]
                    cells.append(f"{x[0]['ms']:.3f}" if x else "")
                else:
                    x = [x for x in gr if x["group_size"] == g and x["reduce_size"] == r]
                    cells.append(f"{x[0]['ms']:.3f}" if x else "")
            out.append(f"| {g} | " + " | ".join(cells) + " |")
        out.append("")
    worst = max(pts, key=lambda r: r["ms"])
    out += [f"times in ms; best: {name_of(best)}: {best['ms']:.3f} ms, {best['gflops']:.0f} GFLOP/s, {best['gbs']:.0f} GB/s of "
            f"minimal bytes = {100 * best['hbm_frac']:.1f} % of the HBM roofline; slowest point: {name_of(worst)}, "
            f"{worst['ms'] / best['ms']:.0f}x the best", ""]
    return out


def other_table(d: dict) -> list[str]:
    """SDDMM, MTTKRP and TTM sweeps: points are (group, strategy) or (group, strategy, schedule)."""
    pts = []
    for x in d["points"]:
        pt = x["point"] if "point" in x else [x["group"], x["strategy"]]
        pts.append((int(pt[0]), pt[1], pt[2] if len(pt) > 2 else None, x))
    best = min(pts, key=lambda r: r[3]["ms"])
    stats = ", ".join(f"{k}={v:,}" if isinstance(v, int) else f"{k}={v:.1f}" for k, v in d["stats"].items())
    out = [f"## {d.get('op', '')} on {d['workload']}  ({stats})", ""]
    schedules = sorted({p[2] for p in pts}, key=lambda v: (v is None, v or ""), reverse=True)
    out += ["| " + ("schedule | " if schedules != [None] else "") + "strategy | " + " | ".join(f"G={g}" for g in G) + " |",
            "|---|" + ("---|" if schedules != [None] else "") + "---|" * len(G)]
    for sc in schedules:
        for stg in ("parallel", "serial"):
            cells = []
            for g in G:
                r = [p for p in pts if (p[0], p[1], p[2]) == (g, stg, sc)]
                cells.append("" if not r else (f"**{r[0][3]['ms']:.3f}**" if r[0] is best else f"{r[0][3]['ms']:.3f}"))
            out.append("| " + (f"{sc} | " if sc else "") + f"{stg} | " + " | ".join(cells) + " |")
    b = best[3]
    out += ["", f"times in ms; best: G={best[0]} {best[1]}{' ' + best[2] if best[2] else ''}: {b['ms']:.3f} ms, {b['gflops']:.0f} GFLOP/s, "
            f"{b['gbs']:.0f} GB/s of minimal bytes = {100 * b['hbm_frac']:.1f} % of the HBM roofline", ""]
    return out


def fixed_against_dynamic(tables: dict, title: str) -> list[str]:
    """tables: workload -> {configuration name -> ms}.  Only configurations every workload has are compared."""
    tags = list(tables)
    common = set(tables[tags[0]])
    for t in tags[1:]:
        common &= set(tables[t])
    best = {t: min(tables[t].values()) for t in tags}

    def geo(k):
        return math.exp(sum(math.log(tables[t][k] / best[t]) for t in tags) / len(tags))

    ranked = sorted(common, key=geo)
    out = [f"### {title}", "",
           "Slowdown of one fixed configuration against the choice per workload (1.00 = the workload's best of ALL its "
           "configurations; geometric mean over the workloads).  Configurations that exist for every workload only.", "",
           "| configuration | geomean slowdown | " + " | ".join(tags) + " |", "|---|---|" + "---|" * len(tags)]
    for k in ranked[:8]:
        out.append(f"| {k} | {geo(k):.3f} | " + " | ".join(f"{tables[t][k] / best[t]:.2f}" for t in tags) + " |")
    out += ["", f"Best fixed configuration: {ranked[0]}; choosing per workload instead gains {geo(ranked[0]):.3f}x (the paper's "
            "Table 5 reports 1.1x to 1.4x for this comparison on its matrices and GPUs).", ""]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("kind", choices=("spmm", "tuner", "other"))
    ap.add_argument("workloads", nargs="+")
    ap.add_argument("--dir", default=".", help="where bench.py wrote the JSON files")
    ap.add_argument("--suffix", default="", help="file names are sweep_W<suffix>.json / tuner_W<suffix>.json")
    ap.add_argument("--title", default=None)
    ap.add_argument("--preamble", default="", help="text (the commands, what was measured) put under the title")
    ap.add_argument("--out", required=True)
    a = ap.parse_args()
    lines = []
    if a.kind == "spmm":
        lines += [f"# {a.title or 'Every point of the space, per workload'}", ""]
        if a.preamble:
            lines += [a.preamble, ""]
        tables = {}
        for w in a.workloads:
            d = json.load(open(os.path.join(a.dir, f"sweep_{w}{a.suffix}.json")))
            lines += spmm_tables(d)
            tables[w] = {name_of(x): x["ms"] for x in d["points"]}
        if len(tables) > 1:
            lines += fixed_against_dynamic(tables, "One fixed point against the choice per workload")
    elif a.kind == "other":
        lines += [f"# {a.title or 'Every point, per workload'}", ""]
        if a.preamble:
            lines += [a.preamble, ""]
        for w in a.workloads:
            lines += other_table(json.load(open(os.path.join(a.dir, f"sweep_{w}{a.suffix}.json"))))
    else:
        lines += [f"# {a.title or 'The tuner over the whole space (sgap_autotune_csr_cfg)'}", ""]
        if a.preamble:
            lines += [a.preamble, ""]
        tables = {}
        for w in a.workloads:
            d = json.load(open(os.path.join(a.dir, f"tuner_{w}{a.suffix}.json")))
            tab = sorted(d["table"], key=lambda r: r["ms"])
            lines += [header(d), "", f"{len(tab)} configurations rated; the ten fastest and the slowest:", "",
                      "| configuration | ms | against the best |", "|---|---|---|"]
            for r in tab[:10] + tab[-1:]:
                lines.append(f"| {name_of(r)} | {r['ms']:.3f} | {r['ms'] / tab[0]['ms']:.2f} |")
            lines.append("")
            tables[w] = {name_of(x): x["ms"] for x in tab}
        if len(tables) > 1:
            lines += fixed_against_dynamic(tables, "One fixed configuration against the tuner's choice per workload")
    with open(a.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print(f"wrote {a.out}")


if __name__ == "__main__":
    main()
