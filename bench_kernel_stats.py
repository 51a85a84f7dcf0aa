"""Turns the kernel trace of a `rocprofv3 --kernel-trace --stats` run of bench.py into the short
table kept under profiles/: per kernel of libactqkv.so the number of launches and the average,
minimum and maximum duration, with launches of one kernel that differ in grid size listed
separately (the two teams of a queued prefill attention are the same kernel with 224 and 32
workgroups; a one-window launch and a 32-window launch of the same kernel are different work).

    python bench_kernel_stats.py --trace <dir>/<prefix>_kernel_trace.csv --title "..." \
        --command "<the rocprofv3 command>" --out profiles/<name>.md [--min-calls 2]
"""
from __future__ import annotations

import argparse
import csv
from collections import defaultdict


def short(name: str) -> str:
    name = name.split("(")[0]
    return name.replace("void ", "").replace("actqkv::", "")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace", required=True)
    ap.add_argument("--title", required=True)
    ap.add_argument("--command", default="")
    ap.add_argument("--out", required=True)
    ap.add_argument("--note", default="")
    args = ap.parse_args()

    groups = defaultdict(list)          # (kernel, workgroups) -> durations in ns
    t_first, t_last, busy = None, None, 0
    with open(args.trace, newline="") as f:
        for row in csv.DictReader(f):
            if "actqkv::" not in row["Kernel_Name"]:
                continue
            t0, t1 = int(row["Start_Timestamp"]), int(row["End_Timestamp"])
            wg = 1
            for ax in "XYZ":
                wg *= max(int(row[f"Grid_Size_{ax}"]) // max(int(row[f"Workgroup_Size_{ax}"]), 1), 1)
            groups[(short(row["Kernel_Name"]), wg)].append(t1 - t0)
            t_first = t0 if t_first is None else min(t_first, t0)
            t_last = t1 if t_last is None else max(t_last, t1)
            busy += t1 - t0
    lines = [f"# {args.title}", ""]
    if args.command:
        lines += ["Command (from /tmp on the GPU box, TMPDIR=/tmp, repository at $GRAFT_REPO_ROOT):", "",
                  "```", args.command, "```", ""]
    lines += ["Kernels of libactqkv.so from the kernel trace, launches of one kernel grouped by their number of "
              "workgroups; durations in microseconds (start to end stamp of the dispatch).", "",
              "| kernel | workgroups | launches | avg us | min us | max us | total ms |",
              "|---|---:|---:|---:|---:|---:|---:|"]
    for (name, wg), d in sorted(groups.items(), key=lambda kv: -sum(kv[1])):
        lines.append(f"| {name} | {wg} | {len(d)} | {sum(d) / len(d) / 1e3:.2f} | {min(d) / 1e3:.2f} | "
                     f"{max(d) / 1e3:.2f} | {sum(d) / 1e6:.2f} |")
    if args.note:
        lines += ["", args.note]
    with open(args.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
