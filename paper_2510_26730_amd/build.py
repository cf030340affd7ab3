"""Build the HIP library in-tree: ``paper_2510_26730_amd/libexpertflow.so`` (gfx950)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libexpertflow.so")
SOURCES = ["ef_api.hip", "ef_route.hip", "ef_ffn.hip", "ef_ffn_tiled.hip", "ef_ffn_q4.hip", "ef_dist.hip"]
HEADERS = ["ef_kernels.h", "ef_device.h", "ef_cache.h", os.path.join("..", "..", "include", "expertflow.h")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result", "-Wno-unknown-attributes"]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    return any(os.path.getmtime(p) > t for p in deps)


def build(force: bool = True, extra_flags=()) -> str:
    """Compile every HIP source for gfx950 and link the shared library."""
    if not force and not is_stale():
        return LIB
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", LIB] + [os.path.join(CSRC, f) for f in SOURCES]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True, extra_flags=sys.argv[1:]))
