#!/usr/bin/env python3
"""Turn the kernel_stats.csv of a `rocprofv3 --kernel-trace --stats` run of bench.py into a short markdown table.

    rocprofv3 --kernel-trace --stats -d DIR -o kt --output-format csv -- python3 bench.py --steps 20 --warmup 3 \\
        --no-cpu-baseline
    python3 -m paper_2605_12396_amd.kt_summary DIR "<title>" "<command line that was profiled>"
"""
import csv
import glob
import os
import sys


def main():
    d, title, cmd = sys.argv[1], sys.argv[2], sys.argv[3]
    files = glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True)
    if not files:
        raise SystemExit("no kernel_stats.csv under %s" % d)
    rows = list(csv.DictReader(open(files[0])))
    print("# rocprofv3 kernel trace: %s\n" % title)
    print("Command (repository root, after `cd /tmp && export TMPDIR=/tmp && cd -`):\n")
    print("    rocprofv3 --kernel-trace --stats -d %s -o kt --output-format csv -- %s" % (d, cmd))
    print("    python3 -m paper_2605_12396_amd.kt_summary %s ...\n" % d)
    print("Durations in ns, all launches of the run (warm-up, timed steps, the per-kernel event pass, set-up calls).\n")
    print("| kernel | calls | average ns | min ns | max ns | % of GPU time |")
    print("|---|---:|---:|---:|---:|---:|")
    for r in rows:
        name = r["Name"].replace("void ", "").replace("nz::", "")
        name = name.split("(")[0] if name.startswith("k_") else name[:90]
        if float(r["Percentage"]) < 0.05:
            continue
        print("| `%s` | %s | %.0f | %s | %s | %s |" % (name, r["Calls"], float(r["AverageNs"]), r["MinNs"], r["MaxNs"], r["Percentage"]))


if __name__ == "__main__":
    main()
