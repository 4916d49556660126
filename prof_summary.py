"""Turn rocprofv3 CSV output into the short text / JSON summaries kept under profiles/.

  python prof_summary.py stats   <dir-of-kernel-trace-run>
  python prof_summary.py traffic <dir-of-FETCH_SIZE-run> <dir-of-WRITE_SIZE-run> \
         --copy-bytes <bytes the calibration copy moved> [--kernel mpq_gemv_kernel]

`stats` prints calls / average / min / max duration per kernel from *_kernel_stats.csv and, for the
product kernel, the same split by grid size from *_kernel_trace.csv.
`traffic` scales the FETCH_SIZE / WRITE_SIZE readings (KiB per dispatch) of the product kernel by
what the same counters read for a plain device-to-device copy of known size in the same run.
"""
import argparse
import collections
import csv
import glob
import json
import os
import sys


def _one(d, pattern):
    hits = sorted(glob.glob(os.path.join(d, "**", pattern), recursive=True))
    if not hits:
        raise SystemExit(f"no {pattern} under {d}")
    return hits[0]


def stats(d, kernel):
    rows = list(csv.DictReader(open(_one(d, "*kernel_stats.csv"))))
    print("kernel, calls, avg_ns, min_ns, max_ns, percent")
    for r in rows:
        print(f"{r['Name'][:90]}, {r['Calls']}, {float(r['AverageNs']):.0f}, {r['MinNs']}, {r['MaxNs']}, {r['Percentage']}")
    by_grid = collections.defaultdict(list)
    for r in csv.DictReader(open(_one(d, "*kernel_trace.csv"))):
        if kernel in r["Kernel_Name"]:
            by_grid[int(r["Grid_Size_X"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    print(f"\n{kernel} by grid size (threads): calls, avg_ns, median_ns, min_ns")
    tot = n = 0
    for g, v in sorted(by_grid.items()):
        v.sort()
        tot += sum(v)
        n += len(v)
        print(f"  grid {g}: {len(v)}, {sum(v) / len(v):.0f}, {v[len(v) // 2]}, {v[0]}")
    if n:
        print(f"  all: {n} launches, average {tot / n:.0f} ns")


def _counter(d, name, kernel):
    mine, copies = [], []
    for r in csv.DictReader(open(_one(d, "*counter_collection.csv"))):
        if r["Counter_Name"] != name:
            continue
        if kernel in r["Kernel_Name"]:
            mine.append(float(r["Counter_Value"]))
        elif "copyBuffer" in r["Kernel_Name"] or "elementwise_kernel" in r["Kernel_Name"] and "copy" in r["Kernel_Name"].lower():
            copies.append(float(r["Counter_Value"]))
    return mine, copies


def traffic(fetch_dir, write_dir, copy_bytes, kernel):
    out = {"kernel": kernel, "copy_bytes": copy_bytes}
    total = 0.0
    for name, d in (("FETCH_SIZE", fetch_dir), ("WRITE_SIZE", write_dir)):
        mine, copies = _counter(d, name, kernel)
        if not mine or not copies:
            raise SystemExit(f"{name}: kernel or calibration copy not found in {d}")
        cal = max(copies)                       # the calibration copy is the largest copy of the run
        factor = copy_bytes / (cal * 1024.0)    # bytes per counted KiB
        per_launch = sum(mine) / len(mine) * 1024.0 * factor
        out[name] = {"launches": len(mine), "mean_kib": sum(mine) / len(mine), "copy_kib": cal,
                     "scale": factor, "bytes_per_launch": per_launch}
        total += per_launch
    out["hbm_bytes_per_launch"] = round(total)
    print(json.dumps(out, indent=1))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    a = sub.add_parser("stats")
    a.add_argument("dir")
    a.add_argument("--kernel", default="mpq_gemv_kernel")
    b = sub.add_parser("traffic")
    b.add_argument("fetch_dir")
    b.add_argument("write_dir")
    b.add_argument("--copy-bytes", type=float, required=True)
    b.add_argument("--kernel", default="mpq_gemv_kernel")
    args = ap.parse_args()
    if args.cmd == "stats":
        stats(args.dir, args.kernel)
    else:
        traffic(args.fetch_dir, args.write_dir, args.copy_bytes, args.kernel)


if __name__ == "__main__":
    sys.exit(main())
