"""Per-kernel durations from a rocprofv3 kernel trace, with the first launches of each kernel set aside.

    rocprofv3 --kernel-trace --output-format csv -d OUT -o run -- python3 -m paper_2504_15465_amd.profile_kernels --what gemm8192 --warm 30 --reps 20
    python3 -m paper_2504_15465_amd.profile_summary OUT/*/run_kernel_trace.csv --skip 30

The clock manager needs some hundred milliseconds of load to settle; `--skip N` lists the first N
dispatches of every kernel apart from the rest, so that the steady-state average can be read off.
Prints a markdown table; reads the CSV only (no GPU needed).
"""
from __future__ import annotations

import argparse
import csv
import re
from collections import OrderedDict


def short(name: str) -> str:
    return re.sub(r"^void ", "", name).replace("lithos::", "")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("trace", help="*_kernel_trace.csv written by rocprofv3 --kernel-trace")
    ap.add_argument("--skip", type=int, default=0, help="dispatches of each kernel listed apart as warm-up")
    ap.add_argument("--grid", type=int, default=0, help="only dispatches with this many workgroups (0: all)")
    ap.add_argument("--by-queue", action="store_true", help="one row per (kernel, hardware queue, workgroups per dispatch): "
                    "tells whole launches from atoms, and one CU-masked queue from another")
    ap.add_argument("--kernel", default="", help="only kernels whose name contains this text")
    args = ap.parse_args()
    rows = OrderedDict()
    with open(args.trace, newline="") as f:
        for r in csv.DictReader(f):
            wg = int(r.get("Workgroup_Size_X") or r.get("Workgroup_Size") or 1)
            gx = int(r.get("Grid_Size_X") or r.get("Grid_Size") or 0)
            blocks = gx // max(1, wg)
            if args.grid and blocks != args.grid:
                continue
            name = short(r["Kernel_Name"])
            if args.kernel and args.kernel not in name:
                continue
            if args.by_queue:
                name = "%s, queue %s, %d workgroups" % (name, r.get("Queue_Id", "?"), blocks)
            rows.setdefault(name, []).append((int(r["Start_Timestamp"]), int(r["End_Timestamp"])))
    print("| kernel | part | launches | avg us | min us | max us |\n|---|---|---|---|---|---|")
    for name, spans in rows.items():
        spans.sort()
        dur = [(e - s) * 1e-3 for s, e in spans]
        for label, part in (("first %d" % args.skip, dur[:args.skip]), ("rest", dur[args.skip:])):
            if part:
                print("| `%s` | %s | %d | %.1f | %.1f | %.1f |" % (name, label, len(part), sum(part) / len(part), min(part), max(part)))


if __name__ == "__main__":
    main()
