"""Turns rocprofv3 CSV output into the short summaries kept under profiles/, and reads them back for bench.py.

    python -m paper_2210_12219_amd.profile_summary --kernel enumerate_paired_kernel --workload headline \\
        --stats DIR_OF_KERNEL_TRACE --counters DIR [DIR ...] --traffic FETCH_DIR WRITE_DIR \\
        --orderings 232243200 --command "..." > profiles/enumerate_paired_headline.md

--stats     a directory written by `rocprofv3 --kernel-trace --stats --output-format csv`
--counters  directories written by `rocprofv3 --pmc ... --output-format csv` (one per pass)
--traffic   two such directories for FETCH_SIZE and WRITE_SIZE, taken with `bench.py --copy-probe`: the counters
            are scaled by what they read for the probe's plain copy kernel (256 MiB read, 256 MiB written)
The summary starts with `key: value` lines (`ppo_version`, `kernel_avg_ns`, `valu_issue`, `traffic_bytes_per_launch`
...) that `read_summary` parses; bench.py quotes them only while the library's version is still the one profiled.
"""
from __future__ import annotations

import argparse
import csv
import glob
import os
import re

PROBE_BYTES = 256 * 1024 * 1024   # bench.py --copy-probe: one kernel that reads and writes this much


def _rows(directory, suffix):
    out = []
    for f in glob.glob(os.path.join(directory, "**", f"*{suffix}"), recursive=True):
        out += list(csv.DictReader(open(f)))
    return out


def kernel_stats(directory, kernel):
    """(calls, average ns, min ns, max ns) of the kernel and the table of all kernels."""
    rows = _rows(directory, "kernel_stats.csv")
    table = [(r["Name"], int(r["Calls"]), float(r["AverageNs"]), float(r["MinNs"]), float(r["MaxNs"]), float(r["Percentage"]))
             for r in rows]
    mine = [x for x in table if kernel in x[0]]
    return (mine[0] if mine else None), table


def counters(directories, kernel):
    """sum over the chip, per dispatch of the kernel, of every counter found (mean over the dispatches seen)."""
    total, calls = {}, {}
    for d in directories:
        per_dispatch = {}
        for r in _rows(d, "counter_collection.csv"):
            if kernel in r["Kernel_Name"]:
                key = (r["Counter_Name"], r["Dispatch_Id"])
                per_dispatch[key] = per_dispatch.get(key, 0.0) + float(r["Counter_Value"])
        for (name, _), v in per_dispatch.items():
            total[name] = total.get(name, 0.0) + v
            calls[name] = calls.get(name, 0) + 1
    return {k: total[k] / calls[k] for k in total}


def traffic(fetch_dir, write_dir, kernel):
    """HBM bytes per launch of the kernel: FETCH_SIZE and WRITE_SIZE scaled by what they read for the copy probe."""
    out = {}
    for name, d in (("FETCH_SIZE", fetch_dir), ("WRITE_SIZE", write_dir)):
        mine, probe, n_mine = 0.0, 0.0, 0
        seen = set()
        for r in _rows(d, "counter_collection.csv"):
            if r["Counter_Name"] != name:
                continue
            if kernel in r["Kernel_Name"]:
                mine += float(r["Counter_Value"])
                seen.add(r["Dispatch_Id"])
            # the probe is torch's in-place elementwise add: the one vectorized_elementwise kernel that is not a fill
            if "vectorized_elementwise_kernel" in r["Kernel_Name"] and "_add<" in r["Kernel_Name"]:
                probe += float(r["Counter_Value"])
        n_mine = max(len(seen), 1)
        factor = PROBE_BYTES / probe if probe else float("nan")   # bytes per count
        out[name] = (mine / n_mine, factor, mine / n_mine * factor)
    return out


def read_summary(path):
    """the `key: value` lines at the top of a summary, as a dict of floats / strings; {} if the file is missing."""
    out = {}
    if not os.path.exists(path):
        return out
    for line in open(path):
        m = re.match(r"^([a-z_0-9]+): (.+)$", line.strip())
        if m:
            try:
                out[m.group(1)] = float(m.group(2))
            except ValueError:
                out[m.group(1)] = m.group(2)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--kernel", required=True)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--ppo-version", type=int, required=True)
    ap.add_argument("--stats")
    ap.add_argument("--counters", nargs="*", default=[])
    ap.add_argument("--traffic", nargs=2)
    ap.add_argument("--orderings", type=float, default=0.0, help="orderings per launch (for per-ordering figures)")
    ap.add_argument("--command", action="append", default=[], help="a command that produced the inputs (repeatable)")
    ap.add_argument("--note", action="append", default=[])
    a = ap.parse_args()
    lines = [f"# {a.kernel}: {a.workload}", ""]
    keys = [("ppo_version", a.ppo_version), ("kernel", a.kernel), ("workload", a.workload)]
    body = []
    if a.stats:
        mine, table = kernel_stats(a.stats, a.kernel)
        if mine:
            keys += [("kernel_calls", mine[1]), ("kernel_avg_ns", mine[2]), ("kernel_min_ns", mine[3]), ("kernel_max_ns", mine[4])]
        body += ["## Kernel trace", "", "| kernel | calls | average ns | min ns | max ns | share % |", "|---|---|---|---|---|---|"]
        body += [f"| `{n[:70]}` | {c} | {avg:,.0f} | {mn:,.0f} | {mx:,.0f} | {pct:.2f} |" for n, c, avg, mn, mx, pct in
                 sorted(table, key=lambda x: -x[5])[:8]]
        body.append("")
    if a.counters:
        c = counters(a.counters, a.kernel)
        if "SQ_BUSY_CYCLES" in c:
            clocks = c["SQ_BUSY_CYCLES"] / 32.0 * 1.0   # summed over 32 shader engines
            keys.append(("busy_clocks", clocks))
            if "SQ_INSTS_VALU" in c:
                # one vector instruction occupies a SIMD for 4 clocks; 256 compute units x 4 SIMDs
                keys.append(("valu_issue", c["SQ_INSTS_VALU"] * 4.0 / (1024.0 * clocks)))
            if "SQ_INSTS_SALU" in c:
                keys.append(("salu_issue", c["SQ_INSTS_SALU"] * 4.0 / (1024.0 * clocks)))
        body += ["## Counters (sums over the chip for one launch)", "", "| counter | value | per ordering |", "|---|---|---|"]
        for name in sorted(c):
            per = f"{c[name] / a.orderings:.4g}" if a.orderings else ""
            body.append(f"| {name} | {c[name]:.5g} | {per} |")
        body.append("")
    if a.traffic:
        t = traffic(a.traffic[0], a.traffic[1], a.kernel)
        total = t["FETCH_SIZE"][2] + t["WRITE_SIZE"][2]
        keys.append(("traffic_bytes_per_launch", total))
        body += ["## HBM traffic", "", "| counter | kernel reads | bytes per count (from the copy probe) | bytes |", "|---|---|---|---|"]
        body += [f"| {k} | {v[0]:.6g} | {v[1]:.5g} | {v[2]:.5g} |" for k, v in t.items()]
        body.append("")
    lines += [f"{k}: {v}" for k, v in keys] + [""]
    if a.command:
        lines += ["Commands (from the repository root on the GPU box, after `cd /tmp && export TMPDIR=/tmp`; `$R` is the root):", ""]
        lines += [f"    {c}" for c in a.command] + [""]
    lines += [n for n in a.note] + ([""] if a.note else [])
    print("\n".join(lines + body))


if __name__ == "__main__":
    main()
