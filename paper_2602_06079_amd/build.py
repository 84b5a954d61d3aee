"""Builds libcanz.so in-tree: host planner with g++, HIP kernels with hipcc for gfx950.

Usage: ``python -m paper_2602_06079_amd.build`` (or ``build()`` from Python).
hipcc cross-compiles without a GPU.  Objects go to ``csrc/_build`` (ignored by git);
the library lands next to this file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OUT = os.path.join(HERE, "libcanz.so")
EXAMPLE_SRC = os.path.join(CSRC, "example_c_abi_step.cpp")
EXAMPLE_OUT = os.path.join(HERE, "c_abi_step")      # a C++ program that uses the C ABI directly, no Python

HOST_SOURCES = ["error.cpp", "partition.cpp", "microgroup.cpp", "tp_schedule.cpp"]
HIP_SOURCES = ["muon_step.hip", "elementwise.hip", "gemm_bf16.hip", "gemm_f32.hip", "shampoo.hip", "soap.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CXX = os.environ.get("CXX", "g++")

# -ffp-contract=off: the partitioner's fp64 decisions must not depend on fused multiply-adds.
HOST_FLAGS = ["-O2", "-fPIC", "-std=c++17", "-ffp-contract=off", "-Wall", "-Wextra", "-I", INCLUDE, "-I", CSRC]
# packed fp32 instructions are switched off for all device code (a hipcc-only flag).
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-I", INCLUDE, "-I", CSRC,
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), proc.stdout))
    return proc.stdout


def build(verbose: bool = False) -> str:
    """Compile every source and link libcanz.so; returns its path."""
    if shutil.which(HIPCC) is None and not os.path.exists(HIPCC):
        raise RuntimeError("hipcc not found at %s" % HIPCC)
    bdir = os.path.join(CSRC, "_build")
    os.makedirs(bdir, exist_ok=True)
    jobs = []
    for src in HOST_SOURCES:
        obj = os.path.join(bdir, src + ".o")
        jobs.append(([CXX] + HOST_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj], obj))
    for src in HIP_SOURCES:
        obj = os.path.join(bdir, src + ".o")
        jobs.append(([HIPCC] + HIP_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj], obj))
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        logs = list(pool.map(lambda j: _run(j[0]), jobs))
    if verbose:
        for (cmd, _), log in zip(jobs, logs):
            print(" ".join(cmd))
            if log.strip():
                print(log)
    tmp = OUT + ".tmp"
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [obj for _, obj in jobs])
    os.replace(tmp, OUT)
    if os.path.exists(EXAMPLE_SRC):
        _run([HIPCC, "-O2", "-std=c++17", "-I", INCLUDE, EXAMPLE_SRC, "-o", EXAMPLE_OUT, "-L", HERE, "-lcanz",
              "-Wl,-rpath,$ORIGIN"])
    return OUT


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
