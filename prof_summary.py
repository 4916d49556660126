"""Turn rocprofv3 CSV output into the short text / JSON summaries kept under profiles/.

  python prof_summary.py stats   <dir-of-kernel-trace-run>
  python prof_summary.py traffic <dir-of-FETCH_SIZE-run> <dir-of-WRITE_SIZE-run> \
         --copy-bytes <bytes the calibration copy moved> [--kernel mpq_gemv_kernel]

`stats` prints calls / average / min / max duration per kernel from *_kernel_stats.csv and, for the
product kernel, the same split by grid size from *_kernel_trace.csv.
`traffic` scales the FETCH_SIZE / WRITE_SIZE readings (KiB per dispatch) of the product kernel by
what the same counters read for a plain device-to-device copy of known size in the same run.

  python prof_summary.py counters <dir-of-a---pmc-run> [<dir> ...] [--kernel mpq_]

`counters` prints the mean of every counter per kernel whose name contains --kernel (the first launches of
a kernel, still cold, are left out) and a few ratios derived from them.
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


def counters(dirs, kernel, skip):
    table = collections.defaultdict(lambda: collections.defaultdict(list))
    for d in dirs:
        for r in csv.DictReader(open(_one(d, "*counter_collection.csv"))):
            if kernel in r["Kernel_Name"]:
                table[r["Kernel_Name"].split("(")[0][:70]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    for k, cs in sorted(table.items()):
        mean = {c: sum(v[skip:]) / max(1, len(v[skip:])) for c, v in cs.items()}
        n = max(len(v) for v in cs.values())
        print(f"{k}: {n} launches (first {skip} left out)")
        for c in sorted(mean):
            print(f"  {c} = {mean[c]:.0f}")
        # SQ_WAVE_CYCLES, SQ_WAIT_INST_ANY, SQ_ACTIVE_INST_* and SQ_INSTS_* count in units of four cycles per wave
        # or per instruction; SQ_BUSY_CYCLES counts cycles on each of the 32 shader engines
        if "SQ_BUSY_CYCLES" in mean and "SQ_ACTIVE_INST_VALU" in mean:
            simds = 1024.0
            print(f"  -> vector ALU busy {100 * 4 * mean['SQ_ACTIVE_INST_VALU'] / simds / (mean['SQ_BUSY_CYCLES'] / 32):.0f} % of the kernel's cycles")
        if "SQ_BUSY_CYCLES" in mean and "SQ_ACTIVE_INST_SCA" in mean:
            print(f"  -> scalar unit busy {100 * 4 * mean['SQ_ACTIVE_INST_SCA'] / 1024.0 / (mean['SQ_BUSY_CYCLES'] / 32):.0f} % of the kernel's cycles")
        if "SQ_WAVE_CYCLES" in mean and "SQ_WAIT_INST_ANY" in mean:
            print(f"  -> waves wait in s_waitcnt {100 * mean['SQ_WAIT_INST_ANY'] / mean['SQ_WAVE_CYCLES']:.0f} % of their time")
        if "SQ_WAVE_CYCLES" in mean and "SQ_BUSY_CYCLES" in mean:
            print(f"  -> resident waves per SIMD, average {4 * mean['SQ_WAVE_CYCLES'] / 1024.0 / (mean['SQ_BUSY_CYCLES'] / 32):.1f}")
        if "SQ_INSTS_VALU" in mean and "SQ_INSTS_SALU" in mean:
            print(f"  -> scalar instructions per vector instruction {mean['SQ_INSTS_SALU'] / mean['SQ_INSTS_VALU']:.2f}")
        if "SQ_LDS_IDX_ACTIVE" in mean and "SQ_LDS_BANK_CONFLICT" in mean and mean["SQ_LDS_IDX_ACTIVE"]:
            print(f"  -> LDS bank conflicts {100 * mean['SQ_LDS_BANK_CONFLICT'] / mean['SQ_LDS_IDX_ACTIVE']:.0f} % of its active cycles")


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
    c = sub.add_parser("counters")
    c.add_argument("dirs", nargs="+")
    c.add_argument("--kernel", default="mpq_")
    c.add_argument("--skip", type=int, default=8)
    args = ap.parse_args()
    if args.cmd == "stats":
        stats(args.dir, args.kernel)
    elif args.cmd == "counters":
        counters(args.dirs, args.kernel, args.skip)
    else:
        traffic(args.fetch_dir, args.write_dir, args.copy_bytes, args.kernel)


if __name__ == "__main__":
    sys.exit(main())
