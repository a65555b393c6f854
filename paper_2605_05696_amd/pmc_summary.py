"""Reduce rocprofv3 --pmc CSV output to per-kernel averages.

usage: python -m paper_2605_05696_amd.pmc_summary [--only=<kernel substring>] <counter_collection.csv> [<more.csv> ...]
       python -m paper_2605_05696_amd.pmc_summary --stats <kernel_stats.csv>

       python -m paper_2605_05696_amd.pmc_summary --traffic <FETCH_SIZE run.csv> <WRITE_SIZE run.csv> <kernel> \
              <algorithmic bytes per launch> <workload text> [out.json]

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


def traffic(fetch_csv, write_csv, kernel, alg_bytes, workload, out_path):
    """HBM bytes per launch of `kernel` from one FETCH_SIZE run and one WRITE_SIZE run, each scaled by
    what the same counter reads for calibrate_copy (1 GiB read, 1 GiB written) in the same run."""
    import json
    f, w = summarise([fetch_csv]), summarise([write_csv])

    def pick(table, counter, name):
        rows = [(k, v) for k, v in table.items() if k[0] == counter and name in k[1]]
        if len(rows) != 1:
            raise SystemExit(f"{counter}: {len(rows)} kernels match {name!r}: {[k[1] for k, _ in rows]}")
        return rows[0][0][1], rows[0][1]
    gib_kib = float(1 << 20)
    _, (_, cal_f, _) = pick(f, "FETCH_SIZE", "calibrate_copy")
    _, (_, cal_w, _) = pick(w, "WRITE_SIZE", "calibrate_copy")
    name, (n_f, kib_f, us_f) = pick(f, "FETCH_SIZE", kernel)
    _, (n_w, kib_w, us_w) = pick(w, "WRITE_SIZE", kernel)
    fs, ws = gib_kib / cal_f, gib_kib / cal_w
    rd, wr = kib_f * 1024.0 * fs, kib_w * 1024.0 * ws
    rec = {"kernel": name, "workload": workload, "dispatches_fetch_run": n_f, "dispatches_write_run": n_w,
           "fetch_size_kib_per_launch": kib_f, "write_size_kib_per_launch": kib_w,
           "calibrate_copy_fetch_kib": cal_f, "calibrate_copy_write_kib": cal_w, "fetch_scale": fs,
           "write_scale": ws, "hbm_read_bytes_per_launch": rd, "hbm_write_bytes_per_launch": wr,
           "hbm_bytes_per_launch": rd + wr, "mean_us_fetch_run": us_f, "mean_us_write_run": us_w}
    if alg_bytes:
        rec["algorithmic_bytes_per_launch"] = alg_bytes
        rec["traffic_over_algorithmic"] = (rd + wr) / alg_bytes
    text = json.dumps(rec, indent=1)
    if out_path:
        with open(out_path, "w") as fh:
            fh.write(text + "\n")
    print(text)
    return 0


def main(argv):
    if len(argv) < 2:
        print(__doc__)
        return 2
    if argv[1] == "--stats":
        return stats_table(argv[2])
    if argv[1] == "--traffic":
        # --traffic <fetch.csv> <write.csv> <kernel substring> <algorithmic bytes per launch or 0> <workload text> [out.json]
        return traffic(argv[2], argv[3], argv[4], float(argv[5]), argv[6], argv[7] if len(argv) > 7 else None)
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
