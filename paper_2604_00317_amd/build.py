"""Compiles the HIP library in-tree: paper_2604_00317_amd/libnimble_plan.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libnimble_plan.so")
SOURCES = ["api.hip", "kernels_stream.hip", "kernels_resident.hip",
           "kernels_persistent.hip", "kernels_alg1.hip", "kernels_post.hip", "kernels_adaptive.hip",
           "host_topo.cpp"]
# -ffp-contract=off: one IEEE operation per statement on host and device (no FMA contraction).
# packed-fp32-ops is switched off for every device compile of this build.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
         "-Wno-unused-command-line-argument"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("NIMBLE_EXTRA_HIPCC_FLAGS", "").split()
    cmd = [hipcc, *FLAGS, *extra, "-shared", "-o", LIB]
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        if s.endswith(".cpp"):
            cmd += ["-x", "hip", src]
        else:
            cmd.append(src)
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
