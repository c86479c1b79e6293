#!/usr/bin/env python3
"""Turns rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench.py into the HBM traffic per launch that
bench.py reports as roofline.traffic.

The two counters read in KiB per dispatch; how a KiB of theirs relates to a KiB moved is calibrated on
the same box with a plain copy of known size (`bench.py --calibrate-copy`: the library's 128-bit copy
kernel over 256 MiB, so 262144 KiB read and 262144 KiB written per dispatch):

    rocprofv3 --pmc FETCH_SIZE -d out/cal_fetch -o p --output-format csv -- python3 bench.py --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d out/cal_write -o p --output-format csv -- python3 bench.py --calibrate-copy
    rocprofv3 --pmc FETCH_SIZE -d out/cfg4_fetch -o p --output-format csv -- python3 bench.py --workload cfg4 --steps 5 --warmup 1 --no-cpu --no-extra
    rocprofv3 --pmc WRITE_SIZE -d out/cfg4_write -o p --output-format csv -- python3 bench.py --workload cfg4 --steps 5 --warmup 1 --no-cpu --no-extra
    python3 bench_traffic.py --workload cfg4 --kernel plane_gemm_kernel --fetch out/cfg4_fetch \\
        --write out/cfg4_write --cal-fetch out/cal_fetch --cal-write out/cal_write

It rewrites the row of that workload in profiles/hbm_traffic.md (a table; bench.py reads the last column).
"""
from __future__ import annotations

import argparse
import csv
import glob
import os
import re

ROOT = os.path.dirname(os.path.abspath(__file__))
TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.md")
CAL_KIB = 262144.0
HEADER = ["workload", "kernel", "dispatches", "FETCH_SIZE KiB", "fetch scale", "WRITE_SIZE KiB", "write scale",
          "bytes per launch"]
INTRO = """# HBM traffic per launch of the dominant kernels (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)

Written by `bench_traffic.py` (its docstring has the commands).  Counter readings are averages over the kernel's
dispatches in KiB; the scale factors come from the same counters' readings for the library's 256 MiB copy kernel
on the same box (262144 KiB read and written per dispatch).  bytes per launch = (FETCH x scale + WRITE x scale) x 1024;
`bench.py` reports it as `roofline.traffic`.

"""


def mean_counter(directory: str, counter: str, kernel_substr: str):
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise SystemExit(f"no counter_collection.csv under {directory}")
    vals = []
    for f in files:
        with open(f, newline="") as fh:
            for r in csv.DictReader(fh):
                if r["Counter_Name"] == counter and kernel_substr in r["Kernel_Name"]:
                    vals.append(float(r["Counter_Value"]))
    if not vals:
        raise SystemExit(f"no {counter} rows for a kernel containing '{kernel_substr}' under {directory}")
    return sum(vals) / len(vals), len(vals)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--kernel", required=True, help="substring of the dominant kernel's name")
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    ap.add_argument("--cal-fetch", required=True)
    ap.add_argument("--cal-write", required=True)
    ap.add_argument("--cal-kernel", default="hbm_copy_kernel")
    a = ap.parse_args()
    cal_f, _ = mean_counter(a.cal_fetch, "FETCH_SIZE", a.cal_kernel)
    cal_w, _ = mean_counter(a.cal_write, "WRITE_SIZE", a.cal_kernel)
    sf, sw = CAL_KIB / cal_f, CAL_KIB / cal_w
    fetch, n = mean_counter(a.fetch, "FETCH_SIZE", a.kernel)
    write, _ = mean_counter(a.write, "WRITE_SIZE", a.kernel)
    nbytes = int(round((fetch * sf + write * sw) * 1024))
    row = [a.workload, a.kernel, str(n), f"{fetch:.1f}", f"{sf:.3f}", f"{write:.1f}", f"{sw:.3f}", str(nbytes)]
    rows = {}
    if os.path.exists(TABLE):
        with open(TABLE) as fh:
            for ln in fh:
                m = re.match(r"\|\s*([\w.-]+)\s*\|", ln)
                if m and m.group(1) != "workload" and not set(m.group(1)) <= {"-"}:
                    rows[m.group(1)] = [c.strip() for c in ln.strip().strip("|").split("|")]
    rows[a.workload] = row
    with open(TABLE, "w") as fh:
        fh.write(INTRO)
        fh.write("| " + " | ".join(HEADER) + " |\n")
        fh.write("|" + "---|" * len(HEADER) + "\n")
        for k in sorted(rows):
            fh.write("| " + " | ".join(rows[k]) + " |\n")
    print(" | ".join(row))


if __name__ == "__main__":
    main()
