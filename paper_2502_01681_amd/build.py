"""Build libdg4.so (HIP kernels + C ABI) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdg4.so")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["dg4_graph.cpp", "dg4_graph_gpu.hip", "dg4_api.cpp", "dg4_kernels.hip", "dg4_sweep.hip", "dg4_flow.hip",
           "dg4_static.hip"]
HEADERS = [os.path.join(CSRC, "dg4_internal.h"), os.path.join(CSRC, "dg4_device.h"), os.path.join(ROOT, "include", "dg4.h")]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in sources() + HEADERS)


def _flags():
    return ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
            # packed fp32 VALU forms are switched off for every kernel of this library
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            # MFMA accumulators in VGPRs: leaves the AGPR half of the register file to the
            # weights that the persistent sweep kernel keeps resident
            "-mllvm", "-amdgpu-mfma-vgpr-form=1",
            # no wave-wide rewriting of atomics: the ticket draws of the persistent kernels are single-lane
            # already, and the rewriting makes the wave wait for the result on the spot
            "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC,
            "-Wall", "-Wno-unused-function"]


def build(force: bool = True) -> str:
    """Compile every source with hipcc for gfx950 (one object per source, in parallel) and link the
    shared library. force=False recompiles only the sources that changed since their object was made."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in HEADERS)

    def compile_one(src):
        obj = os.path.join(OBJ, os.path.basename(src) + ".o")
        if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header):
            return obj
        subprocess.check_call([hipcc] + _flags() + ["-c", src, "-o", obj], stderr=subprocess.DEVNULL if os.environ.get("DG4_QUIET") else None)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, sources()))
    subprocess.check_call([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(force="--incremental" not in sys.argv))
