"""Turns two rocprofv3 counter runs of `bench.py --pmc-pass` (one with --pmc FETCH_SIZE, one
with --pmc WRITE_SIZE, CSV output) into HBM bytes per kernel dispatch.

Each counter is scaled by what it reads for the library's plain copy kernel of known size,
which runs first in such a pass.  Writes a short text summary and updates bench_traffic.json
next to this file, which bench.py reports as roofline.traffic as long as the kernels' sources
are the ones the counters were taken with (a hash of csrc/ is stored with the bytes).

    python bench_traffic.py --workload c3_128k \
        --fetch <dir>/f_counter_collection.csv --write <dir>/w_counter_collection.csv \
        --info <dir>/pmc_pass_c3_128k.json --summary profiles/<name>.md \
        --command "<how the CSVs were made>"

--info is the file the counter pass itself wrote: the configuration of the pass, the mean
number of blocks it selected and the algorithmic bytes of its launches.
"""
from __future__ import annotations

import argparse
import csv
import hashlib
import json
import os
from collections import defaultdict

HERE = os.path.dirname(os.path.abspath(__file__))


def source_hash() -> str:
    """Hash of the kernels' sources: the stored traffic is only reported for these."""
    d = os.path.join(HERE, "paper_2502_13542_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(d, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


ATTENTION = {
    "c3_128k": ("attn_prefill_mfma_queued_kernel", ["attn_prefill_mfma_queued_kernel"]),
    "c4_decode": ("attn_decode_select_kernel", ["attn_decode_select_kernel"]),
}
OURS = ("probe_", "score_", "select_", "attn_", "append_", "cutoff_", "decode_", "gather_")


def short(name: str) -> str:
    name = name.split("(")[0]
    return name.replace("void ", "").replace("actqkv::", "").split("<")[0]


def per_kernel(path: str, counter: str):
    """kernel -> list of counter values, one per dispatch (rows of one dispatch are added up)."""
    disp = defaultdict(float)
    names = {}
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            if row["Counter_Name"] != counter:
                continue
            key = int(row["Dispatch_Id"])
            disp[key] += float(row["Counter_Value"])
            names[key] = short(row["Kernel_Name"])
    out = defaultdict(list)
    for key in sorted(disp):
        out[names[key]].append(disp[key])
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True, choices=sorted(ATTENTION))
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--copy-bytes", type=int, default=256 << 20)
    ap.add_argument("--summary", required=True)
    ap.add_argument("--command", default="")
    ap.add_argument("--info", default="", help="the JSON file bench.py --pmc-pass wrote for this pass")
    ap.add_argument("--calls", type=int, default=0,
                    help="attention calls in the pass, if a call is more than one dispatch of the kernel "
                         "(two teams of workgroups); default: one call per dispatch")
    args = ap.parse_args()

    fetch, write = per_kernel(args.fetch, "FETCH_SIZE"), per_kernel(args.write, "WRITE_SIZE")
    if "copy_bytes_kernel" not in fetch or "copy_bytes_kernel" not in write:
        raise SystemExit("no copy_bytes_kernel dispatch in the counter files")
    f_copy, w_copy = fetch["copy_bytes_kernel"][0], write["copy_bytes_kernel"][0]
    f_scale, w_scale = args.copy_bytes / f_copy, args.copy_bytes / w_copy   # bytes per counter unit

    lines = [f"# HBM traffic per dispatch, {args.workload} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)", ""]
    if args.command:
        lines += ["Commands:", "", "```", args.command, "```", ""]
    lines += [f"Calibration: copy_bytes_kernel moves {args.copy_bytes} bytes each way; FETCH_SIZE read "
              f"{f_copy:.0f}, WRITE_SIZE read {w_copy:.0f} -> {f_scale:.1f} and {w_scale:.1f} bytes per "
              f"counter unit (1024 = the counters' nominal KiB).", "",
              "| kernel | dispatches | fetch MB / dispatch | write MB / dispatch |", "|---|---|---|---|"]
    for name in sorted(set(fetch) | set(write)):
        if name == "copy_bytes_kernel" or not any(k in name for k in OURS):
            continue
        fv, wv = fetch.get(name, []), write.get(name, [])
        n = max(len(fv), len(wv), 1)
        lines.append(f"| {name} | {n} | {sum(fv) * f_scale / n / 1e6:.3f} | {sum(wv) * w_scale / n / 1e6:.3f} |")

    main_kernel, parts = ATTENTION[args.workload]
    launches = len(fetch.get(main_kernel, []))
    if launches == 0:
        raise SystemExit(f"no {main_kernel} dispatch in the counter files")
    if args.calls > 0:
        launches = args.calls
    f_bytes = sum(sum(fetch.get(k, [])) for k in parts) * f_scale / launches
    w_bytes = sum(sum(write.get(k, [])) for k in parts) * w_scale / launches
    lines += ["", f"Attention call ({' + '.join(parts)}), mean over {launches} calls: "
                  f"fetch {f_bytes / 1e6:.3f} MB, write {w_bytes / 1e6:.3f} MB."]
    info = {}
    if args.info:
        with open(args.info) as f:
            info = json.load(f)
        lines += ["", "The pass these counters were taken on (written by the pass itself):", ""]
        lines += [f"* {k}: {v}" for k, v in sorted(info.items())]
        if "algorithmic_bytes_per_launch" in info:
            a = float(info["algorithmic_bytes_per_launch"])
            lines += ["", f"Algorithmic bytes per launch at this pass's selection (reads and writes): "
                          f"{a / 1e6:.3f} MB; (fetched + written) / algorithmic = {(f_bytes + w_bytes) / a:.3f}."]
    os.makedirs(os.path.dirname(os.path.abspath(args.summary)), exist_ok=True)
    with open(args.summary, "w") as f:
        f.write("\n".join(lines) + "\n")

    jpath = os.path.join(HERE, "bench_traffic.json")
    try:
        with open(jpath) as f:
            data = json.load(f)
    except (OSError, ValueError):
        data = {}
    data[args.workload] = {"fetch_bytes_per_launch": f_bytes, "write_bytes_per_launch": w_bytes,
                           "launches": launches, "fetch_scale": f_scale, "write_scale": w_scale,
                           "kernels": parts, "source_hash": source_hash(), "pass": info}
    with open(jpath, "w") as f:
        json.dump(data, f, indent=1, sort_keys=True)
        f.write("\n")
    print("\n".join(lines))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
