"""Build libfbx.so (HIP kernels + C++ host side) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libfbx.so")
SOURCES = ["fbx_plan.cpp", "fbx_api.cpp", "fbx_jit.cpp", "fbx_support.hip", "fbx_walk.hip", "fbx_tile.hip", "fbx_clean.hip"]
HEADERS = ["fbx_internal.h", "fbx_device.h", "fbx_arena.h", "fbx_split.h", os.path.join(_ROOT, "include", "fbx.h")]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def command() -> list:
    return [
        hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
        # keep the compiler from forming packed-FP32 instructions anywhere
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        # atomics whose one lane asks for a work item stay plain: rewritten as a wavefront-wide
        # reduction they would wait for the answer at once instead of where it is used
        "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
        "-x", "hip",
    ] + (["-DFBX_TILE_PROF"] if os.environ.get("FBX_TILE_PROF") else []) + [
        "-I", os.path.join(_ROOT, "include"), "-I", CSRC,
        "-o", LIB,
    ] + [os.path.join(CSRC, s) for s in SOURCES] + ["-ldl"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + [h if os.path.isabs(h) else os.path.join(CSRC, h) for h in HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if force or stale():
        cmd = command()
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print(LIB)
