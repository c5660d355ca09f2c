"""Build libdg4.so (HIP kernels + C ABI) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdg4.so")
SOURCES = ["dg4_graph.cpp", "dg4_graph_gpu.hip", "dg4_api.cpp", "dg4_kernels.hip", "dg4_sweep.hip"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + [os.path.join(CSRC, "dg4_internal.h"), os.path.join(CSRC, "dg4_device.h"), os.path.join(ROOT, "include", "dg4.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True) -> str:
    """Compile every source with hipcc for gfx950 and link the shared library."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
           "-x", "hip",
           # packed fp32 VALU forms are switched off for every kernel of this library
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           # MFMA accumulators in VGPRs: leaves the AGPR half of the register file to the
           # weights that the persistent sweep kernel keeps resident
           "-mllvm", "-amdgpu-mfma-vgpr-form=1",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-Wall", "-Wno-unused-function",
           "-o", LIB] + sources()
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
