"""Builds libnmconv1d.so (the HIP library behind include/nm_conv1d.h) in-tree for gfx950."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_PKG, "csrc")
OBJ_DIR = os.path.join(_PKG, "_build")
LIB_PATH = os.path.join(_PKG, "libnmconv1d.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose: bool = False) -> str:
    """Compile every .hip source (one hipcc process per file, side by side) and link them into one
    shared library; returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    jobs = []
    for src in sources():
        obj = os.path.join(OBJ_DIR, os.path.splitext(os.path.basename(src))[0] + ".o")
        jobs.append((src, obj, [hipcc] + HIPCC_FLAGS + ["-c", "-o", obj, src]))

    def run(job):
        if verbose:
            print(" ".join(job[2]), flush=True)
        subprocess.run(job[2], check=True)
        return job[1]

    with ThreadPoolExecutor(max_workers=min(8, max(len(jobs), 1))) as pool:
        objs = list(pool.map(run, jobs))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", LIB_PATH] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
