#!/usr/bin/env python3
"""Turn two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, then WRITE_SIZE) into HBM bytes per kernel launch.

    rocprofv3 --pmc FETCH_SIZE -d DIR_F -o pmc --output-format csv -- python3 bench.py --steps 3 --warmup 1 \\
        --no-cpu-baseline --calib-copy 3
    rocprofv3 --pmc WRITE_SIZE -d DIR_W -o pmc --output-format csv -- python3 bench.py ... (same)
    python3 -m paper_2605_12396_amd.pmc_summary DIR_F DIR_W 268435456 c2

Both counters are reported in KiB per dispatch.  They are scaled by what the same counter reads for the plain
elementwise copy kernel of `--calib-copy` (which reads and writes exactly copy_bytes), so that systematic
over- or under-counting of the counter cancels.  Output: one line per kernel, `<workload> <stage>/<kernel>
fetch_bytes write_bytes`, the format bench.py reads, plus the calibration factors as comments.
"""
import collections
import csv
import glob
import os
import sys

KERNELS = [("k_stats<0, 0, 0>", ["compress/stats"]), ("k_codebook", ["compress/codebook", "reduce/codebook", "reduce_local/codebook"]),
           ("k_encode<0, 0, 0>", ["compress/encode"]), ("k_encode<1, 0, 0>", ["reduce/encode", "reduce_local/encode"]),
           ("k_decode<0, 256, 0>", ["decompress/decode"]), ("k_decode_finish", ["decompress/finish"]),
           ("k_decode<1, 256, 0>", ["reduce/stage_a"]), ("k_decode<2, 512, 0>", ["reduce/add_b"]),
           ("k_decode<3, 512, 0>", ["reduce_local/add_local"]), ("k_fix", ["reduce/fix", "reduce_local/fix", "reduce_local_rea/fix"]),
           ("k_encode<2, 0, 0>", ["compress_rea/encode"]),
           ("k_rea_finish", ["compress_rea/finish", "reduce_local_rea/finish"]),
           ("k_decode<5, 512, 0>", ["reduce_local_rea/add_local"]), ("k_encode<3, 0, 0>", ["reduce_local_rea/encode"])]


def per_kernel(d, counter):
    files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no counter_collection.csv under %s" % d)
    agg = collections.defaultdict(list)
    for fn in files:
        for r in csv.DictReader(open(fn)):
            if r["Counter_Name"] == counter:
                agg[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return agg


def pick(agg, needle):
    vals = [v for k, vs in agg.items() if needle in k for v in vs]
    return vals


def main():
    d_f, d_w, copy_bytes, workload = sys.argv[1], sys.argv[2], float(sys.argv[3]), sys.argv[4]
    fetch, write = per_kernel(d_f, "FETCH_SIZE"), per_kernel(d_w, "WRITE_SIZE")

    def copy_kernel(agg):
        # the calibration kernel is torch's elementwise add: the largest-traffic kernel that is not ours
        cand = {k: sum(v) / len(v) for k, v in agg.items() if "nz::" not in k and "elementwise" in k}
        if not cand:
            raise SystemExit("no calibration copy kernel found (run bench.py with --calib-copy)")
        k = max(cand, key=cand.get)
        return cand[k]
    cf, cw = copy_kernel(fetch), copy_kernel(write)
    sf, sw = copy_bytes / (cf * 1024.0), copy_bytes / (cw * 1024.0)
    print("# calibration: copy kernel of %d bytes each way read FETCH_SIZE=%.0f KiB, WRITE_SIZE=%.0f KiB "
          "-> scale %.4f / %.4f" % (copy_bytes, cf, cw, sf, sw))
    for needle, names in KERNELS:
        f, w = pick(fetch, needle), pick(write, needle)
        if not f or not w:
            continue
        fb, wb = sf * 1024.0 * sum(f) / len(f), sw * 1024.0 * sum(w) / len(w)
        for nm in names:
            print("%s %s %.0f %.0f" % (workload, nm, fb, wb))


if __name__ == "__main__":
    main()
