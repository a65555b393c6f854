"""Reduce rocprofv3 --pmc CSV output to per-kernel averages.

usage: python -m paper_2605_05696_amd.pmc_summary [--only=<kernel substring>] <counter_collection.csv> [<more.csv> ...]
       python -m paper_2605_05696_amd.pmc_summary --stats <kernel_stats.csv>

The second form shortens the per-kernel table ``rocprofv3 --kernel-trace --stats
--output-format csv`` writes (calls, average / min / max duration in us, share).

Prints, per counter and kernel, the number of dispatches, the mean counter value
per dispatch and the mean dispatch duration (counters serialise the kernels).  FETCH_SIZE and WRITE_SIZE are reported by the hardware in
KiB; the plain copy kernel ``calibrate_copy`` moves a known number of bytes, so
the ratio (known bytes) / (counted KiB * 1024) calibrates the counters.
"""
from __future__ import annotations

import csv
import sys
from collections import defaultdict


def summarise(paths):
    acc = defaultdict(lambda: [0, 0.0, 0.0])
    for path in paths:
        with open(path, newline="") as f:
            for row in csv.DictReader(f):
                name = row.get("Kernel_Name") or row.get("kernel_name") or ""
                counter = row.get("Counter_Name") or row.get("counter_name") or ""
                value = float(row.get("Counter_Value") or row.get("counter_value") or 0.0)
                short = name.split("(")[0].replace("void ", "")
                a = acc[(counter, short)]
                a[0] += 1
                a[1] += value
                try:
                    a[2] += (float(row["End_Timestamp"]) - float(row["Start_Timestamp"])) / 1e3
                except (KeyError, ValueError):
                    pass
    return {k: (n, total / n, us / n) for k, (n, total, us) in acc.items() if n}


def stats_table(path, top=24):
    with open(path, newline="") as f:
        rows = list(csv.DictReader(f))
    print(f"{'kernel':72s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'pct':>6s}")
    for row in rows[:top]:
        print(f"{row['Name'][:72]:72s} {int(row['Calls']):6d} {float(row['AverageNs']) / 1e3:10.2f} "
              f"{float(row['MinNs']) / 1e3:10.2f} {float(row['MaxNs']) / 1e3:10.2f} {float(row['Percentage']):6.2f}")
    return 0


def main(argv):
    if len(argv) < 2:
        print(__doc__)
        return 2
    if argv[1] == "--stats":
        return stats_table(argv[2])
    table = summarise([a for a in argv[1:] if not a.startswith("--")])
    only = [a[7:] for a in argv[1:] if a.startswith("--only=")]
    print(f"{'counter':40s} {'kernel':40s} {'dispatches':>10s} {'mean per dispatch':>20s} {'mean us':>10s}")
    for (counter, kernel), (n, mean, us) in sorted(table.items()):
        if only and not any(o in kernel for o in only):
            continue
        print(f"{counter:40s} {kernel[:40]:40s} {n:10d} {mean:20.1f} {us:10.1f}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
