"""Sums the hardware counters of rocprofv3 --pmc runs of `bench.py --pmc-pass` over the dispatches of
one kernel and writes the short table kept under profiles/ (counter values per attention call), with
the figures derived from them: matrix-core busy share, LDS bytes per cycle, where the wavefronts'
time goes.

    python bench_counters.py --kernel attn_prefill_mfma_queued_kernel --calls 8 --title "..." \
        --command "<the rocprofv3 commands>" --out profiles/<name>.md <run a>/p_counter_collection.csv <run b>/...
"""
from __future__ import annotations

import argparse
import csv
from collections import defaultdict

CUS, SIMDS, XCDS = 256, 1024, 8


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("csv", nargs="+")
    ap.add_argument("--kernel", required=True)
    ap.add_argument("--calls", type=int, required=True, help="calls of the entry point in the pass")
    ap.add_argument("--cus", type=int, default=CUS, help="compute units the kernel's first launch fills")
    ap.add_argument("--title", required=True)
    ap.add_argument("--command", default="")
    ap.add_argument("--note", default="")
    ap.add_argument("--out", required=True)
    args = ap.parse_args()

    tot = defaultdict(float)
    disp = defaultdict(set)
    for path in args.csv:
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                if args.kernel in row["Kernel_Name"]:
                    tot[row["Counter_Name"]] += float(row["Counter_Value"])
                    disp[row["Counter_Name"]].add(row["Dispatch_Id"])
    n = args.calls
    lines = [f"# {args.title}", ""]
    if args.command:
        lines += ["Commands (from /tmp on the GPU box, TMPDIR=/tmp; one counter group per run):", "", "```",
                  args.command, "```", ""]
    lines += [f"Sums over the dispatches of {args.kernel} in one pass, divided by the {n} calls of the pass "
              f"({len(next(iter(disp.values()), ()))} dispatches).", "",
              "| counter | per call |", "|---|---:|"]
    lines += [f"| {k} | {tot[k] / n:,.0f} |" for k in sorted(tot)]
    lines.append("")
    g = lambda k: tot.get(k, 0.0) / n
    if g("SQ_INSTS_MFMA") and g("SQ_VALU_MFMA_BUSY_CYCLES"):
        lines.append(f"* Matrix-core instructions per call: {g('SQ_INSTS_MFMA'):,.0f} (wavefront level; 32x32x16 bf16: "
                     f"{g('SQ_INSTS_MFMA') * 32 * 32 * 16 * 2 / 1e9:.1f} GFLOP issued); busy cycles per instruction "
                     f"{g('SQ_VALU_MFMA_BUSY_CYCLES') / g('SQ_INSTS_MFMA'):.1f}.")
    if g("GRBM_GUI_ACTIVE") and g("SQ_VALU_MFMA_BUSY_CYCLES"):
        act = g("GRBM_GUI_ACTIVE") / XCDS
        util = g("SQ_VALU_MFMA_BUSY_CYCLES") / (SIMDS * act)
        lines.append(f"* GRBM_GUI_ACTIVE is counted per XCD: {act:,.0f} active cycles per call on each of the {XCDS}.  "
                     f"Matrix-core busy cycles / ({SIMDS} SIMDs x active cycles) = {100 * util:.1f} % of the chip"
                     + (f", {100 * util * CUS / args.cus:.1f} % of the {args.cus} compute units of the first launch"
                        if args.cus != CUS else "") + ".")
        if g("SQ_INSTS_LDS"):
            lines.append(f"* LDS instructions per call: {g('SQ_INSTS_LDS'):,.0f} (1 KB operand reads almost all of "
                         f"them): {g('SQ_INSTS_LDS') * 1024 / (act * args.cus):.0f} bytes per active cycle and "
                         f"compute unit in use; bank conflict cycles {g('SQ_LDS_BANK_CONFLICT'):,.0f}.")
    if g("SQ_WAVE_CYCLES"):
        w = g("SQ_WAVE_CYCLES")
        lines.append(f"* Wavefront time (SQ_WAVE_CYCLES): waiting (SQ_WAIT_ANY) {100 * g('SQ_WAIT_ANY') / w:.0f} %, "
                     f"issuing (SQ_ACTIVE_INST_ANY) {100 * g('SQ_ACTIVE_INST_ANY') / w:.0f} %, of which vector ALU "
                     f"including matrix-core issue (SQ_ACTIVE_INST_VALU) {100 * g('SQ_ACTIVE_INST_VALU') / w:.0f} %.")
    if args.note:
        lines += ["", args.note]
    with open(args.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
