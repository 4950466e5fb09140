"""Short text summaries of rocprofv3 CSV output (the tables kept under profiles/).

    python -m paper_2605_01106_amd.rocprof_summary stats <dir> [--top N]
        per-kernel statistics of a `rocprofv3 --kernel-trace --stats --output-format csv` run
        (reads <dir>/**/*kernel_stats.csv): a markdown table.

    python -m paper_2605_01106_amd.rocprof_summary counter <dir> [--copy-kib K]
        one `rocprofv3 --pmc <COUNTER> --output-format csv` run (reads <dir>/**/*counter_collection.csv):
        the counter's mean value per dispatch for every kernel, as JSON.  With --copy-kib the
        calibration factor K / (mean value of the device-to-device copy kernels of K KiB) is added:
        `bench.py --counters` ends with four copies of 262144 KiB for this purpose.

Both print to stdout; the raw files can be large and stay where rocprofv3 wrote them.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import sys


def _find(directory: str, pattern: str) -> str:
    hits = sorted(glob.glob(os.path.join(directory, "**", pattern), recursive=True))
    if not hits:
        sys.exit(f"no {pattern} under {directory}")
    return hits[0]


def stats(directory: str, top: int) -> None:
    rows = list(csv.DictReader(open(_find(directory, "*kernel_stats.csv"))))
    total = sum(int(r["TotalDurationNs"]) for r in rows)
    print(f"{len(rows)} kernels, {sum(int(r['Calls']) for r in rows)} dispatches, {total / 1e6:.1f} ms of kernel time\n")
    print("| kernel | calls | total ms | avg us | min us | max us | % |")
    print("|---|---|---|---|---|---|---|")
    for r in rows[:top]:
        print(f"| `{r['Name']}` | {r['Calls']} | {int(r['TotalDurationNs']) / 1e6:.2f} | {float(r['AverageNs']) / 1e3:.2f} | "
              f"{int(r['MinNs']) / 1e3:.2f} | {int(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.2f} |")


def counter(directory: str, copy_kib: float) -> None:
    path = _find(directory, "*counter_collection.csv")
    acc = collections.defaultdict(lambda: [0, 0.0])
    copies = collections.defaultdict(list)            # per-dispatch values of the copy kernels (calibration)
    name = None
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            name = r["Counter_Name"]
            a = acc[r["Kernel_Name"]]
            a[0] += 1
            a[1] += float(r["Counter_Value"])
            if "copy" in r["Kernel_Name"].lower():
                copies[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    out = {"counter": name, "file": os.path.basename(path),
           "mean_per_dispatch": {k: {"dispatches": n, "mean": s / n} for k, (n, s) in sorted(acc.items(), key=lambda kv: -kv[1][1])}}
    if copy_kib > 0:
        # the calibration copies are the largest copies of the run: average the dispatches within a factor 2 of the largest
        out["calibration"] = {}
        for k, vals in copies.items():
            big = [v for v in vals if v >= 0.5 * max(vals)]
            m = sum(big) / len(big)
            out["calibration"][k] = {"dispatches": len(big), "mean": m, "factor": copy_kib / m if m > 0 else None}
    print(json.dumps(out, indent=1))


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats")
    s.add_argument("dir")
    s.add_argument("--top", type=int, default=40)
    c = sub.add_parser("counter")
    c.add_argument("dir")
    c.add_argument("--copy-kib", type=float, default=0.0)
    args = ap.parse_args()
    if args.cmd == "stats":
        stats(args.dir, args.top)
    else:
        counter(args.dir, args.copy_kib)


if __name__ == "__main__":
    main()
