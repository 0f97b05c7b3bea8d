"""Builds libegeria.so (the gfx950 kernels and their C-ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libegeria.so")
SOURCES = ["api.hip", "quantize.hip", "gemm_i8.hip", "gram.hip", "bert.hip", "freeze.hip", "cache.hip", "cast.hip"]
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
                        os.path.join(os.path.dirname(HERE), "include", "egeria.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build_library(force: bool = True) -> str:
    """Compile every HIP source for gfx950 into paper_2201_06227_amd/libegeria.so."""
    if not force and not is_stale():
        return LIB
    cmd = [HIPCC] + FLAGS + ["-o", LIB] + sources()
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    return LIB
