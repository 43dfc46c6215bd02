#!/usr/bin/env python3
"""Turn one rocprofv3 --pmc run of bench.py with SQ counters into per-kernel instruction figures.

    rocprofv3 --pmc SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS \\
        SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS -d DIR -o pmc --output-format csv -- \\
        python3 bench.py --steps 2 --warmup 1 --no-cpu-baseline
    python3 -m paper_2605_12396_amd.sq_summary DIR 67108864

(eight SQ counters are what one pass holds).  Per kernel of the library, averaged over its launches:
wave-level VALU / SALU / LDS instructions per symbol of the message (the counters count wavefront instructions, a
wavefront covers 64 lanes, so `per symbol` = instructions x 64 / symbols), and the share of the SIMD cycles of the
kernel's busy time that issue VALU work: a wave64 VALU instruction occupies its SIMD for 4 cycles, the chip has 1024
SIMDs, and SQ_BUSY_CYCLES comes summed over the 32 shader engines, so share = 4 x SQ_INSTS_VALU / (SQ_BUSY_CYCLES / 32
x 1024) = SQ_INSTS_VALU / (8 x SQ_BUSY_CYCLES).
"""
import collections
import csv
import glob
import os
import sys


def main():
    d, symbols = sys.argv[1], float(sys.argv[2])
    files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no counter_collection.csv under %s" % d)
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for fn in files:
        for r in csv.DictReader(open(fn)):
            k = r["Kernel_Name"]
            if "nz::" not in k:
                continue
            agg[k.replace("nz::", "").split("(")[0].replace("void ", "")][r["Counter_Name"]].append(float(r["Counter_Value"]))
    print("# kernel  launches  VALU/symbol  SALU/symbol  LDS/symbol  VALU-issue share of SIMD cycles  waves")
    for k in sorted(agg):
        c = {n: sum(v) / len(v) for n, v in agg[k].items()}
        if c.get("SQ_WAVES", 0) < 1024:             # the small bookkeeping kernels say nothing per symbol
            continue
        per = lambda n: c.get(n, 0.0) * 64.0 / symbols
        share = c.get("SQ_INSTS_VALU", 0.0) / (8.0 * max(c.get("SQ_BUSY_CYCLES", 1.0), 1.0))
        print("%-28s %3d  %6.1f  %6.1f  %6.1f  %5.2f  %d" % (k, len(agg[k]["SQ_WAVES"]), per("SQ_INSTS_VALU"), per("SQ_INSTS_SALU"),
                                                         per("SQ_INSTS_LDS"), share, int(c.get("SQ_WAVES", 0))))


if __name__ == "__main__":
    main()
