"""Condenses rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2501_13986_amd.profsum stats   <dir-with-*_kernel_stats.csv>  "<command>"  > profiles/<name>.txt
  python -m paper_2501_13986_amd.profsum traffic <fetch-dir> <write-dir> "<command>"          > profiles/hbm_traffic_step_f32.txt

`traffic` scales FETCH_SIZE / WRITE_SIZE (KiB per dispatch) by what the same counters read for the
1 GiB device copy that `bench.py --calib-copy` runs, and prints one line per kernel:
"kernel fetch_bytes write_bytes" (bytes per launch), which bench.py reads back.
"""
from __future__ import annotations

import csv
import glob
import os
import sys


def _find(d, pat):
    hits = glob.glob(os.path.join(d, "**", pat), recursive=True)
    if not hits:
        raise SystemExit(f"no {pat} under {d}")
    return hits[0]


def stats(d, cmd):
    rows = list(csv.DictReader(open(_find(d, "*kernel_stats.csv"))))
    print(f"# rocprofv3 --kernel-trace --stats summary (per-kernel, durations in microseconds)")
    print(f"# command: {cmd}")
    print(f"# {'kernel':58s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'total_ms':>10s} {'pct':>6s}")
    for r in rows:
        name = r["Name"]
        if len(name) > 58:
            name = name[:55] + "..."
        print(f"  {name:58s} {int(r['Calls']):6d} {float(r['AverageNs'])/1e3:10.1f} {float(r['MinNs'])/1e3:10.1f} "
              f"{float(r['MaxNs'])/1e3:10.1f} {float(r['TotalDurationNs'])/1e6:10.2f} {float(r['Percentage']):6.2f}")


def _per_kernel(d, counter):
    agg = {}
    for r in csv.DictReader(open(_find(d, "*counter_collection.csv"))):
        if r["Counter_Name"] == counter:
            agg.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return agg


def traffic(dfetch, dwrite, cmd):
    f, w = _per_kernel(dfetch, "FETCH_SIZE"), _per_kernel(dwrite, "WRITE_SIZE")
    copy = [k for k in f if "copyBuffer" in k]
    if not copy:
        raise SystemExit("no device-copy kernel found (run bench.py with --calib-copy)")
    gib = float(1 << 20)   # KiB in the 1 GiB the copy moves each way
    sf = gib / sum(f[copy[0]])
    sw = gib / sum(w[copy[0]])
    print("# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (two runs)")
    print(f"# command: {cmd}")
    print(f"# counters are KiB per dispatch; scaled by the 1 GiB device copy of the same run: fetch x{sf:.3f}, write x{sw:.3f}")
    print("# kernel fetch_bytes write_bytes launches")
    for k in sorted(f):
        if k.startswith("cgtp_"):
            fb = sum(f[k]) / len(f[k]) * 1024 * sf
            wb = sum(w.get(k, [0])) / max(1, len(w.get(k, [0]))) * 1024 * sw
            print(f"{k} {fb:.0f} {wb:.0f} {len(f[k])}")


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "stats":
        stats(sys.argv[2], sys.argv[3])
    elif len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        raise SystemExit(__doc__)
