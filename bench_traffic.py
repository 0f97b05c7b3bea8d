#!/usr/bin/env python3
"""Turns two `rocprofv3 --pmc` runs of bench.py into HBM bytes per kernel launch.

    cd /tmp && export TMPDIR=/tmp && cd <repo>
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d out/pmc_fetch -o f -- \\
        python3 bench.py --workload N --no-others --no-cpu --steps 20 --warmup 3 --calibrate
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d out/pmc_write -o w -- \\
        python3 bench.py --workload N --no-others --no-cpu --steps 20 --warmup 3 --calibrate
    python3 bench_traffic.py --workload N --fetch out/pmc_fetch/f_counter_collection.csv \\
        --write out/pmc_write/w_counter_collection.csv

FETCH_SIZE and WRITE_SIZE are reported in KiB per dispatch.  Each is scaled by
what the same counter reads for bench.py's calibration launches, a scaled
copy of known size (dequantize_kernel: 64 MiB read, 256 MiB written), so that
the figures are bytes that reached HBM as that copy's bytes do.  The result
is appended to profiles/hbm_traffic.txt, one line per kernel:

    cfgN kernel fetch_bytes write_bytes launches source_digest

bench.py reports the entry as roofline.traffic as long as the digest still
matches the kernel's sources.
"""
from __future__ import annotations

import argparse
import csv
import os
import re
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
CAL_READ = float(64 << 20)
CAL_WRITE = float(256 << 20)


def per_kernel(path, counter):
    """kernel short name -> list of counter values (KiB), one per dispatch."""
    out = {}
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter or "egeria::" not in r["Kernel_Name"]:
                continue
            name = r["Kernel_Name"].split("egeria::")[1].split("<")[0].split("(")[0]
            # the GEMM kernel's last two template arguments are the operand type and whether the launch also
            # normalises its rows: only the plain int8 launches belong to the GEMM class of the workload's step
            # (bench.py also times float16 / float32 reference legs, and prices the normalising launch with
            # the layer norms)
            if name == "gemm_i8_kernel" and not re.search(r"gemm_i8_kernel<[^>]*, 0, false>", r["Kernel_Name"]):
                continue
            out.setdefault(name, []).append(float(r["Counter_Value"]))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, required=True)
    ap.add_argument("--fetch", required=True)
    ap.add_argument("--write", required=True)
    args = ap.parse_args()
    import bench
    fetch = per_kernel(args.fetch, "FETCH_SIZE")
    write = per_kernel(args.write, "WRITE_SIZE")
    if "dequantize_kernel" not in fetch or "dequantize_kernel" not in write:
        sys.exit("no calibration launches in the counter files (run bench.py with --calibrate)")
    mean = lambda v: sum(v) / len(v)
    f_scale = CAL_READ / (mean(fetch["dequantize_kernel"]) * 1024.0)
    w_scale = CAL_WRITE / (mean(write["dequantize_kernel"]) * 1024.0)
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    keep = []
    if os.path.exists(path):
        keep = [l for l in open(path) if l.startswith("#") or (l.split() and l.split()[0] != f"cfg{args.workload}")]
    if not any(l.startswith("#") for l in keep):
        keep.insert(0, "# HBM bytes per kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench.py, "
                       "scaled by a copy of known size; written by bench_traffic.py (its docstring has the commands)\n"
                       "# workload kernel fetch_bytes write_bytes launches_averaged source_digest "
                       "| calibration: counter KiB -> bytes factors\n")
    lines = []
    for k in sorted(bench.KERNEL_SOURCES):
        if k in fetch and k in write:
            fb, wb = mean(fetch[k]) * 1024.0 * f_scale, mean(write[k]) * 1024.0 * w_scale
            lines.append(f"cfg{args.workload} {k} {fb:.0f} {wb:.0f} {min(len(fetch[k]), len(write[k]))} "
                         f"{bench.source_digest(k)} | fetch x{f_scale:.4f} write x{w_scale:.4f}\n")
            print(lines[-1], end="")
    with open(path, "w") as f:
        f.writelines(keep + lines)


if __name__ == "__main__":
    main()
