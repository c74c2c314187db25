"""Summarise rocprofv3 CSV output for this library's kernels.

usage:
  python3 rocprof_summary.py stats  <dir>                 # --kernel-trace --stats run
  python3 rocprof_summary.py pmc    <fetch_dir> <write_dir> [--json out.json --workload c4]
  python3 rocprof_summary.py counters <dir> [<dir> ...]   # any --pmc runs: mean per dispatch

`stats` prints calls / average / total duration per kernel from *kernel_stats.csv (or from
*kernel_trace.csv if the stats file is absent).  `pmc` reads *counter_collection.csv of a
FETCH_SIZE run and of a WRITE_SIZE run (both counters are in KiB per dispatch), scales each by
what the same counter reads for the library's copy_kernel on a known number of bytes, and
prints HBM bytes per launch for every kernel.
"""
from __future__ import annotations

import csv
import glob
import json
import os
import sys
from collections import defaultdict

COPY_PROBE_BYTES = 256 << 20


def _find(directory: str, suffix: str):
    hits = sorted(glob.glob(os.path.join(directory, "**", f"*{suffix}"), recursive=True))
    return hits


def short(name: str) -> str:
    name = name.replace("void ", "")
    for key in ("fused_packed_kernel", "fused_kernel", "fold_in_kernel", "reduce_scatter_kernel", "exchange_sum_kernel", "all_gather_kernel",
                "combine_kernel", "copy_kernel", "fill_zero_kernel", "empty_kernel"):
        if key in name:
            args = name[name.find(key) + len(key):]
            args = args[:args.find(">") + 1] if args.startswith("<") else ""
            return key + args
    return name[:70]


def stats(directory: str) -> str:
    rows = []
    files = _find(directory, "kernel_stats.csv")
    if files:
        for f in files:
            for r in csv.DictReader(open(f)):
                rows.append((short(r["Name"]), int(r["Calls"]), float(r["TotalDurationNs"]),
                             float(r["AverageNs"]), float(r["MinNs"]), float(r["MaxNs"])))
    else:
        acc = defaultdict(list)
        for f in _find(directory, "kernel_trace.csv"):
            for r in csv.DictReader(open(f)):
                acc[short(r["Kernel_Name"])].append(float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
        for k, v in acc.items():
            rows.append((k, len(v), sum(v), sum(v) / len(v), min(v), max(v)))
    rows.sort(key=lambda r: -r[2])
    out = [f"{'kernel':58s} {'calls':>7s} {'avg us':>10s} {'min us':>10s} {'max us':>10s} {'total ms':>10s}"]
    for name, calls, total, avg, lo, hi in rows:
        out.append(f"{name:58s} {calls:7d} {avg / 1e3:10.2f} {lo / 1e3:10.2f} {hi / 1e3:10.2f} {total / 1e6:10.2f}")
    return "\n".join(out)


def _counter_per_kernel(directory: str, counter: str):
    acc = defaultdict(list)
    for f in _find(directory, "counter_collection.csv"):
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] == counter:
                acc[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return acc


def pmc(fetch_dir: str, write_dir: str):
    fetch = _counter_per_kernel(fetch_dir, "FETCH_SIZE")
    write = _counter_per_kernel(write_dir, "WRITE_SIZE")
    lines, result = [], {}
    scale = {}
    for label, table in (("FETCH_SIZE", fetch), ("WRITE_SIZE", write)):
        probe = table.get("copy_kernel")
        if not probe:
            raise SystemExit(f"no copy_kernel dispatch in the {label} run: cannot scale the counter")
        avg = sum(probe) / len(probe)
        scale[label] = COPY_PROBE_BYTES / (avg * 1024.0)
        lines.append(f"{label}: copy_kernel of {COPY_PROBE_BYTES} B reads {avg:.1f} KiB per dispatch "
                     f"-> scale factor {scale[label]:.4f} (true bytes / counted bytes)")
    lines.append("")
    lines.append(f"{'kernel':58s} {'launches':>8s} {'fetch MB':>12s} {'write MB':>12s} {'total MB':>12s}")
    for k in sorted(set(fetch) | set(write)):
        f = sum(fetch.get(k, [0])) / max(len(fetch.get(k, [0])), 1) * 1024.0 * scale["FETCH_SIZE"]
        w = sum(write.get(k, [0])) / max(len(write.get(k, [0])), 1) * 1024.0 * scale["WRITE_SIZE"]
        result[k] = {"fetch_bytes": f, "write_bytes": w, "launches": len(fetch.get(k, []))}
        lines.append(f"{k:58s} {len(fetch.get(k, [])):8d} {f / 1e6:12.2f} {w / 1e6:12.2f} {(f + w) / 1e6:12.2f}")
    return "\n".join(lines), result, scale


def counters(directories) -> str:
    """Mean value per dispatch of every counter found, per kernel (library kernels only)."""
    acc = defaultdict(lambda: defaultdict(list))
    for d in directories:
        for f in _find(d, "counter_collection.csv"):
            for r in csv.DictReader(open(f)):
                acc[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    names = sorted({c for k in acc.values() for c in k})
    out = [f"{'kernel':40s} {'dispatches':>10s} " + " ".join(f"{c:>26s}" for c in names)]
    for k in sorted(acc):
        if not any(key in k for key in ("fused", "copy_kernel", "_kernel<")):
            continue
        n = max(len(v) for v in acc[k].values())
        out.append(f"{k:40s} {n:10d} " + " ".join(
            f"{(sum(acc[k][c]) / len(acc[k][c]) if acc[k].get(c) else float('nan')):26.1f}" for c in names))
    return "\n".join(out)


def main(argv) -> int:
    if len(argv) >= 3 and argv[1] == "counters":
        print(counters(argv[2:]))
        return 0
    if len(argv) >= 3 and argv[1] == "stats":
        print(stats(argv[2]))
        return 0
    if len(argv) >= 4 and argv[1] == "pmc":
        text, result, scale = pmc(argv[2], argv[3])
        print(text)
        if "--json" in argv:
            out = argv[argv.index("--json") + 1]
            workload = argv[argv.index("--workload") + 1] if "--workload" in argv else "c4"
            fused = [v for k, v in result.items() if k.startswith("fused_kernel")]
            if fused:
                best = max(fused, key=lambda v: v["launches"])
                json.dump({"workload": workload, "kernel": "fused_kernel",
                           "bytes_per_launch": best["fetch_bytes"] + best["write_bytes"],
                           "fetch_bytes": best["fetch_bytes"], "write_bytes": best["write_bytes"],
                           "scale": scale}, open(out, "w"), indent=1)
        return 0
    print(__doc__)
    return 2


if __name__ == "__main__":
    sys.exit(main(sys.argv))
