"""Builds ``libcgx.so`` (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcgx.so")
OBJ = os.path.join(HERE, "_build")
# (source, object name, extra flags): the quantize kernel is built for chunks of 1024 and of 2048 elements
SOURCES = [("cgx_plan.cpp", "cgx_plan", []), ("cgx_api.cpp", "cgx_api", []), ("cgx_adaptive.cpp", "cgx_adaptive", []),
           ("cgx_quantize.hip", "cgx_quantize_g2", ["-DCGX_GROUPS=2"]),
           ("cgx_quantize.hip", "cgx_quantize_g4", ["-DCGX_GROUPS=4"]),
           ("cgx_reduce.hip", "cgx_reduce_g2", ["-DCGX_GROUPS=2"]),
           ("cgx_reduce.hip", "cgx_reduce_g4", ["-DCGX_GROUPS=4"]), ("cgx_fused.hip", "cgx_fused", []), ("cgx_stats.hip", "cgx_stats", []),
           ("cgx_probe.hip", "cgx_probe", [])]

# -ffp-contract=off: the code decision is binary32 without fused operations.
# packed-fp32 instructions stay disabled for this target.
# kernarg preload: the dispatcher puts the first 16 dwords of a kernel's arguments into scalar registers, so a
# wave's first scalar load is its tile descriptor (0.5 us per launch of 20 us); firmware without the feature
# runs the loads of the compiler's compatibility prologue instead.
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-kernarg-preload-count=16",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unused-function"]


def build(verbose: bool = False, extra=(), jobs: int = 8) -> str:
    """Compiles every source (in parallel: the kernel files take a minute each) and links."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(item):
        src, name, flags = item
        obj = os.path.join(OBJ, name + ".o")
        cmd = [hipcc, *FLAGS, *flags, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True, cwd=CSRC)
        return obj

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True, cwd=CSRC)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
