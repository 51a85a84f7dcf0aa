"""Turns the kernel trace of a `rocprofv3 --kernel-trace --stats` run of bench.py into the short
table kept under profiles/: per kernel of libactqkv.so the number of launches and the average,
minimum and maximum duration.  Kernels named with --split are listed per number of workgroups
(the two teams of a queued prefill attention are the same kernel with 224 and 32 workgroups; a
one-window launch and a 32-window launch of the same kernel are different work).  With
--bench-json (the line the traced bench.py printed) the table is followed by the cross-check of
the line's roofline entry against the trace: the same algorithmic work divided by the trace's
average duration of the dominant kernel.

    python bench_kernel_stats.py --trace <dir>/<prefix>_kernel_trace.csv --title "..." \
        --command "<the rocprofv3 command>" --out profiles/<name>.md \
        [--split attn_prefill_mfma_queued_kernel] [--bench-json <file>] [--dominant <kernel>:<workgroups>]
"""
from __future__ import annotations

import argparse
import csv
import json
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
    ap.add_argument("--split", action="append", default=[],
                    help="kernel name (substring) whose launches are listed per number of workgroups")
    ap.add_argument("--bench-json", default="", help="the JSON line of the traced bench.py run")
    ap.add_argument("--section", default="", help="key of the bench line that holds the roofline entry "
                                                  "(\"decode\" for the decode step; default: the line itself)")
    ap.add_argument("--dominant", default="", help="<kernel substring>:<workgroups> of the roofline's kernel")
    args = ap.parse_args()

    groups = defaultdict(list)          # (kernel, workgroups or 0) -> durations in ns
    with open(args.trace, newline="") as f:
        for row in csv.DictReader(f):
            if "actqkv::" not in row["Kernel_Name"]:
                continue
            t0, t1 = int(row["Start_Timestamp"]), int(row["End_Timestamp"])
            wg = 1
            for ax in "XYZ":
                wg *= max(int(row[f"Grid_Size_{ax}"]) // max(int(row[f"Workgroup_Size_{ax}"]), 1), 1)
            name = short(row["Kernel_Name"])
            if not any(s in name for s in args.split):
                wg = 0
            groups[(name, wg)].append(t1 - t0)
    lines = [f"# {args.title}", ""]
    if args.command:
        lines += ["Command (from /tmp on the GPU box, TMPDIR=/tmp, repository at $GRAFT_REPO_ROOT):", "",
                  "```", args.command, "```", ""]
    lines += ["Kernels of libactqkv.so from the kernel trace; durations in microseconds (start to end stamp of "
              "the dispatch); \"workgroups\" is given where launches of one kernel are listed per launch shape.", "",
              "| kernel | workgroups | launches | avg us | min us | max us | total ms |",
              "|---|---:|---:|---:|---:|---:|---:|"]
    for (name, wg), d in sorted(groups.items(), key=lambda kv: -sum(kv[1])):
        lines.append(f"| {name} | {wg if wg else 'any'} | {len(d)} | {sum(d) / len(d) / 1e3:.2f} | "
                     f"{min(d) / 1e3:.2f} | {max(d) / 1e3:.2f} | {sum(d) / 1e6:.2f} |")
    if args.bench_json:
        with open(args.bench_json) as f:
            line = json.loads(f.read().strip().splitlines()[-1])
        sec = line[args.section] if args.section else line
        rf = sec["roofline"]
        step = (f"ms_per_step {sec['ms_per_step']:.3f}" if "ms_per_step" in sec else
                f"{sec['metric']} {sec['value']:.1f}")
        lines += ["", f"The traced run's own line: {step}; roofline: "
                      f"{rf['achieved']:.1f} {rf['unit']} = {rf['frac']:.4f} of {rf['peak']:.0f}, from an average "
                      f"launch of {rf['avg_launch_us']:.1f} us by HIP events."]
        if args.dominant:
            kname, kwg = args.dominant.rsplit(":", 1)
            d = [x for (n, wg), v in groups.items() if kname in n and (wg == int(kwg) or int(kwg) == 0) for x in v]
            if d:
                # the trace holds the same launches plus those of warm-up, capture and the event pass
                avg = sum(d) / len(d) / 1e3
                work = rf["achieved"] * rf["avg_launch_us"]          # work per launch in unit x us
                shape = f"{kwg} workgroups" if int(kwg) else "every launch shape"
                lines += [f"By the trace: {len(d)} launches of {kname} ({shape}) average {avg:.1f} us "
                          f"-> {work / avg:.1f} {rf['unit']} = {work / avg / rf['peak']:.4f} of peak for the "
                          f"same algorithmic work per launch."]
    if args.note:
        lines += ["", args.note]
    with open(args.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
