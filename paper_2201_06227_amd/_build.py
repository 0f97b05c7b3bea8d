"""Builds libegeria.so (the gfx950 kernels and their C-ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libegeria.so")
SOURCES = ["api.hip", "quantize.hip", "gemm_i8.hip", "gram.hip", "bert.hip", "freeze.hip", "cache.hip", "cast.hip", "affine.hip", "microbench.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # the epilogues' fp32 operation order is part of the contract: no contraction
    "-ffp-contract=off",
    # do not form packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the epilogues index their accumulator arrays with fully unrolled loops (up to 4 x 4 x 16
    # iterations of a long body); at the default limit the largest tile's loops stay rolled and
    # its accumulators end up in scratch memory
    "-mllvm", "-pragma-unroll-threshold=200000",
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "common.hpp"),
                        os.path.join(os.path.dirname(HERE), "include", "egeria.h"),
                        os.path.join(os.path.dirname(HERE), "include", "egeria_profile.h"), os.path.join(CSRC, "gelu_table.inc")]
    return any(os.path.getmtime(d) > t for d in deps)


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + proc.stdout)


def build_library(force: bool = True) -> str:
    """Compile every HIP source for gfx950 and link paper_2201_06227_amd/libegeria.so.  The sources
    are independent translation units (no device code calls across them), compiled side by side.
    force=False recompiles only the sources that are newer than their object files."""
    if not force and not is_stale():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    jobs = []
    headers = [os.path.join(CSRC, "common.hpp"), os.path.join(os.path.dirname(HERE), "include", "egeria.h"),
               os.path.join(os.path.dirname(HERE), "include", "egeria_profile.h"), os.path.join(CSRC, "gelu_table.inc")]
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        fresh = os.path.exists(obj) and all(os.path.getmtime(d) <= os.path.getmtime(obj) for d in [src] + headers)
        jobs.append(([HIPCC] + compile_flags + ["-c", src, "-o", obj], obj, force or not fresh))
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        list(pool.map(lambda j: _run(j[0]) if j[2] else None, jobs))
    _run([HIPCC, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB] + [j[1] for j in jobs])
    return LIB
