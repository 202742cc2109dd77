"""Build libamap.so (HIP kernels + host composer + C ABI) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libamap.so")

SOURCES = ["amap_compose.cpp", "amap_graph.cpp", "amap_layout.cpp", "amap_host.cpp", "amap_plan.cpp", "amap_plan_check.cpp", "amap_kernels.hip",
           "amap_gemm.hip"]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
    # The piece kernel reads its by-value argument block through many inlined
    # bodies.  Past a fixed number of uses the optimiser stops reading the
    # block in place and copies all of it to private memory (3 KB of scratch
    # per lane, every field access a scratch load); lift that limit.
    "-mllvm", "-instcombine-max-copied-from-constant-users=100000",
    "-Rpass-analysis=kernel-resource-usage",
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
    usage = kernel_usage(r.stderr)
    after_remark = False
    for line in r.stderr.splitlines():
        if "packed-fp32-ops' is not a recognized feature" in line:
            continue
        if "kernel-resource-usage" in line:
            after_remark = True
            continue
        if after_remark and line.split("|")[0].strip().isdigit() or (after_remark and line.strip().startswith("|")):
            continue  # the source excerpt under a remark
        after_remark = False
        print(line, file=sys.stderr)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    if verbose:
        for name, u in usage.items():
            print(f"{name}: {u}", file=sys.stderr)
    spilled = {n: u for n, u in usage.items() if u.get("ScratchSize [bytes/lane]", 0) != 0}
    if spilled:
        os.remove(LIB)
        raise RuntimeError(f"kernels use scratch memory (argument block copied or registers spilled): {spilled}")
    return LIB


def kernel_usage(stderr: str) -> dict:
    """Per-kernel register / scratch figures from the compiler's resource remarks."""
    usage, cur = {}, None
    for line in stderr.splitlines():
        if "remark:" not in line:
            continue
        body = line.split("remark:", 1)[1].split("[-Rpass-analysis")[0].strip()
        if body.startswith("Function Name:"):
            cur = usage.setdefault(body.split(":", 1)[1].strip(), {})
        elif cur is not None and ":" in body:
            k, v = body.rsplit(":", 1)
            try:
                cur[k.strip()] = int(v)
            except ValueError:
                pass
    return usage


if __name__ == "__main__":
    print(build_lib(verbose=True))
