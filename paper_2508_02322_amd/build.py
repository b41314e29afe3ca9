"""Builds libcamera_hip.so (the C-ABI HIP library) and libcamera_bench.so (machine probes for benchmark
reports) in-tree with hipcc for gfx950.

    python -m paper_2508_02322_amd.build

Each .hip file is compiled to an object in parallel, then linked.  Objects and
the library land next to this file; they are git-ignored.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcamera_hip.so")
BENCH_LIB = os.path.join(HERE, "libcamera_bench.so")
SOURCES = ["api.hip", "route.hip", "bucket.hip", "gemm.hip", "norm.hip", "rank.hip", "gather.hip", "forward.hip",
           "compact.hip"]
BENCH_SOURCES = ["probe.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # keep packed-fp32 instruction selection off for every device function
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{res.stdout}\n{res.stderr}")
    warnings = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if "warning" in warnings:
        sys.stderr.write(warnings + "\n")
    return obj


def _link(lib: str, objs) -> None:
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)}\n{res.stdout}\n{res.stderr}")


def build(verbose: bool = True) -> str:
    every = SOURCES + BENCH_SOURCES
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(every))) as pool:
        objs = list(pool.map(_compile, every))
    _link(LIB, objs[:len(SOURCES)])
    _link(BENCH_LIB, objs[len(SOURCES):])
    if verbose:
        print(f"built {LIB} and {BENCH_LIB}")
    return LIB


if __name__ == "__main__":
    build()
