"""Compiles the HIP library in-tree: paper_2604_00317_amd/libnimble_plan.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libnimble_plan.so")
SOURCES = ["api.hip", "kernels_stream.hip", "kernels_resident.hip",
           "kernels_persistent.hip", "kernels_alg1.hip", "kernels_post.hip", "kernels_adaptive.hip", "kernels_probe.hip",
           "host_topo.cpp"]
# -ffp-contract=off: one IEEE operation per statement on host and device (no FMA contraction).
# packed-fp32-ops is switched off for every device compile of this build.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
         "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compiles every source to an object file (side by side, `jobs` at a time) and links them."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("NIMBLE_EXTRA_HIPCC_FLAGS", "").split()
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(s: str) -> str:
        src = os.path.join(CSRC, s)
        obj = os.path.join(objdir, os.path.splitext(s)[0] + ".o")
        cmd = [hipcc, *FLAGS, *extra, "-c", "-o", obj]
        cmd += ["-x", "hip", src] if s.endswith(".cpp") else [src]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
