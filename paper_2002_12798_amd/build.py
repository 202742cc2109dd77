"""Build libamap.so (HIP kernels + host composer + C ABI) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libamap.so")

SOURCES = ["amap_compose.cpp", "amap_host.cpp", "amap_plan.cpp", "amap_plan_check.cpp", "amap_kernels.hip", "amap_gemm.hip"]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def build_lib(verbose: bool = False, extra=()) -> str:
    cmd = ["hipcc", *FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".hip") else ["-x", "c++", path])
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    # the host pass of hipcc prints one harmless "not a recognized feature"
    # line per function for the packed-fp32 switch; drop those, keep the rest
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    for line in r.stderr.splitlines():
        if "packed-fp32-ops' is not a recognized feature" not in line:
            print(line, file=sys.stderr)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
