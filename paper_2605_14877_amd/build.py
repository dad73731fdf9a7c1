"""Builds the two shared libraries for gfx950 with hipcc: libheatkv.so (HIP kernels + host planner + C ABI of
include/heatkv.h) and libheatkv_probe.so (the measurement aids of include/heatkv_probe.h, for bench.py)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libheatkv.so")
PROBE_LIB = os.path.join(HERE, "libheatkv_probe.so")
LIBRARIES = {LIB: ["plan.cpp", "abi.cpp", "attend.hip", "append.hip", "calibrate.hip"], PROBE_LIB: ["probe.hip"]}
SOURCES = [src for srcs in LIBRARIES.values() for src in srcs]

# Packed-fp32 VALU forms are switched off for every device translation unit.
HIP_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = True) -> str:
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src + ".o")
        cmd = ["hipcc", *HIP_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l or "error" in l)
        if out.strip() and verbose:
            print(out)
        if pr.returncode != 0:
            failed = True
            print(f"compile failed: {src}", file=sys.stderr)
    if failed:
        raise RuntimeError("hipcc failed")
    for lib, srcs in LIBRARIES.items():
        cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib,
               *[os.path.join(HERE, "_build", src + ".o") for src in srcs]]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
