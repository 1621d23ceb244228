"""Condenses rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2501_13986_amd.profsum stats   <dir-with-*_kernel_stats.csv>  "<command>"  > profiles/<name>.txt
  python -m paper_2501_13986_amd.profsum traffic <fetch-dir> <write-dir> "<command>"          > profiles/hbm_traffic_step_f32.txt
  python -m paper_2501_13986_amd.profsum table   <bench-json-line-file> "<command>"           > profiles/bench_all_configs_table.txt
  python -m paper_2501_13986_amd.profsum counters <dir-with-*_counter_collection.csv> "<command>" > profiles/<name>_counters.txt

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


def table(path, cmd):
    """The `kernels` rows of a `bench.py --extra` JSON line as a fixed-width text table."""
    import json
    d = json.loads(open(path).read().strip().splitlines()[-1])
    print("# Per-configuration timings on one MI355X (HIP events on the launch stream, median of 10 after 3 warm-ups;")
    print("# step/* rows: average over the timed steps).  Entry-point times: conv rows include the row-merge kernel and")
    print("# (backward) the receiver-lookup kernel, atomic rows the zero fill.  frac_hbm = algorithmic bytes / 8000 GB/s;")
    print("# binding/frac: the roofline that binds (hbm, alu = 78.6 TFLOP/s plain-FMA vector peak on nonzero FLOPs, mfma =")
    print("# 157.3 TFLOP/s fp32 matrix peak); nocache = fraction of 8000 GB/s when every gathered row counts as HBM bytes.")
    print(f"# command: {cmd}")
    print(f"# {'row':52s} {'dtype':5s} {'ms':>9s} {'GFLOP/s':>10s} {'alg GB/s':>9s} {'frac_hbm':>8s} {'binding':>7s} {'frac':>6s} {'nocache':>7s} {'note'}")
    for r in d["kernels"]:
        note = ""
        if "speedup_vs_seven_dispatches" in r:
            note = f"seven dispatches: {r['seven_dispatch_ms']} ms, fused is {r['speedup_vs_seven_dispatches']}x faster"
        nc = r.get("frac_hbm_nocache", "")
        print(f"  {r['name']:52s} {r['dtype']:5s} {r['ms']:9.4f} {r.get('gflops', 0):10.1f} {r['alg_gbs']:9.1f} {r['frac_hbm']:8.3f} "
              f"{r['binding']:>7s} {r['frac_binding']:6.3f} {str(nc):>7s} {note}")
    print(f"# headline: value={d['value']} {d['unit']}, ms_per_step={d['ms_per_step']}, roofline={d['roofline']}")
    print(f"# cpu_baseline={d['cpu_baseline']}")


def counters(d, cmd):
    """Mean value per dispatch of every collected counter, for the library's own kernels."""
    agg = {}
    for r in csv.DictReader(open(_find(d, "*counter_collection.csv"))):
        if r["Kernel_Name"].startswith("cgtp"):
            agg.setdefault((r["Kernel_Name"], r["Counter_Name"]), []).append(float(r["Counter_Value"]))
    print("# rocprofv3 --pmc summary: mean counter value per dispatch (SQ counters are summed over the chip)")
    print(f"# command: {cmd}")
    print(f"# {'kernel':44s} {'counter':30s} {'dispatches':>10s} {'mean':>16s}")
    for (k, c), v in sorted(agg.items()):
        name = k if len(k) <= 44 else k[:41] + "..."
        print(f"  {name:44s} {c:30s} {len(v):10d} {sum(v) / len(v):16.0f}")


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
    elif len(sys.argv) >= 4 and sys.argv[1] == "counters":
        counters(sys.argv[2], sys.argv[3])
    elif len(sys.argv) >= 4 and sys.argv[1] == "table":
        table(sys.argv[2], sys.argv[3])
    elif len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        raise SystemExit(__doc__)
