"""HBM bytes per launch of the GEMM kernel from rocprofv3 counter runs, as a tracked text table.

bench.py reports `roofline.traffic` from profiles/hbm_traffic_streamk_gemm_kernel.txt; this script writes
that file.  Per workload it needs two counter runs of bench.py (rocprofv3 collects FETCH_SIZE and WRITE_SIZE
in separate runs) and, once, the same two runs of a plain 1 GiB device copy, which calibrate what one unit
of each counter is worth in bytes:

    rocprofv3 --pmc FETCH_SIZE -d out/fetch_cfg5 -o out --output-format csv -- python3 bench.py --workload cfg5 --policy 0 --steps 5 --warmup 2 --no-cpu-baseline
    rocprofv3 --pmc WRITE_SIZE -d out/write_cfg5 -o out --output-format csv -- python3 bench.py --workload cfg5 --policy 0 --steps 5 --warmup 2 --no-cpu-baseline
    rocprofv3 --pmc FETCH_SIZE -d out/fetch_copy -o out --output-format csv -- python3 bench.py --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d out/write_copy -o out --output-format csv -- python3 bench.py --calibrate-copy
    python3 -m paper_2408_11417_amd.hbm_traffic --runs out --library-commit $(git rev-parse --short HEAD) \\
        --entry cfg5:DP --out profiles/hbm_traffic_streamk_gemm_kernel.txt

Each --entry NAME:POLICY[,POLICY...] reads out/fetch_NAME and out/write_NAME (several policy names for one
run: policies that are the same schedule on that workload, e.g. all seven on whole waves of tiles).  The counters are in KiB per dispatch.
The calibration factor is (bytes the copy moves) / (bytes the counter reports for the copy kernel).
CPU only; reads CSV files, nothing else.
"""
import argparse
import csv
import glob
import os
import sys

COPY_BYTES = float(1 << 30)     # bench.py --calibrate-copy reads 1 GiB and writes 1 GiB per copy kernel


def counter_per_dispatch(run_dir, counter, kernel_substr, biggest=False):
    """Mean counter value over the dispatches of the kernels whose name contains kernel_substr (the
    first such dispatch dropped when there are several: it runs cold); with biggest=True over the
    dispatches whose value is within 10 % of the largest one of any kernel (the copy kernel)."""
    files = glob.glob(os.path.join(run_dir, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit("no counter_collection.csv under %s" % run_dir)
    vals = []
    for f in files:
        for row in csv.DictReader(open(f)):
            if row["Counter_Name"] != counter:
                continue
            if biggest or kernel_substr in row["Kernel_Name"]:
                vals.append(float(row["Counter_Value"]))
    if not vals:
        raise SystemExit("counter %s / kernel %s not found under %s" % (counter, kernel_substr, run_dir))
    if biggest:
        top = max(vals)
        vals = [v for v in vals if v >= 0.9 * top]
    elif len(vals) > 1:
        vals = vals[1:]
    return sum(vals) / len(vals)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--runs", required=True, help="folder holding fetch_NAME / write_NAME / fetch_copy / write_copy run folders")
    ap.add_argument("--entry", action="append", default=[], help="NAME:POLICY[,POLICY...], e.g. cfg5:DP (repeatable)")
    ap.add_argument("--library-commit", default="unknown")
    ap.add_argument("--out", required=True)
    args = ap.parse_args()
    kib = 1024.0
    f_copy = counter_per_dispatch(os.path.join(args.runs, "fetch_copy"), "FETCH_SIZE", "", biggest=True) * kib
    w_copy = counter_per_dispatch(os.path.join(args.runs, "write_copy"), "WRITE_SIZE", "", biggest=True) * kib
    f_scale, w_scale = COPY_BYTES / f_copy, COPY_BYTES / w_copy
    lines = ["# HBM bytes per launch of streamk_gemm_kernel (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, KiB per dispatch,",
             "# scaled by what the same counter reads for a plain 1 GiB device copy: fetch x %.3f, write x %.3f);" % (f_scale, w_scale),
             "# written by paper_2408_11417_amd/hbm_traffic.py; library commit %s" % args.library_commit,
             "# workload policy fetch_bytes write_bytes"]
    for e in args.entry:
        name, _, policy = e.partition(":")
        f = counter_per_dispatch(os.path.join(args.runs, "fetch_" + name), "FETCH_SIZE", "streamk_gemm_kernel") * kib * f_scale
        w = counter_per_dispatch(os.path.join(args.runs, "write_" + name), "WRITE_SIZE", "streamk_gemm_kernel") * kib * w_scale
        for pol in policy.split(","):
            lines.append("%s %s %.4g %.4g" % (name, pol, f, w))
    with open(args.out, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print("\n".join(lines))
    return 0


if __name__ == "__main__":
    sys.exit(main())
