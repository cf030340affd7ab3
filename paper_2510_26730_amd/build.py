"""Build the HIP library in-tree: ``paper_2510_26730_amd/libexpertflow.so`` (gfx950)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libexpertflow.so")
SOURCES = ["ef_api.hip", "ef_runtime.hip", "ef_plan.hip", "ef_static.hip", "ef_route.hip", "ef_ffn.hip", "ef_ffn_tiled.hip", "ef_ffn_shared.hip", "ef_ffn_q4.hip", "ef_dist.hip", "ef_calib.hip", "ef_forest.cpp"]
HEADERS = ["ef_ctx.h", "ef_kernels.h", "ef_device.h", "ef_cache.h", "ef_tiled_pipeline.h", os.path.join("..", "..", "include", "expertflow.h")]
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
    """Compile every HIP source for gfx950 (one compiler process per source, in parallel) and link the
    shared library."""
    if not force and not is_stale():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]

    def compile_one(src: str) -> str:
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        subprocess.check_call([HIPCC, *compile_flags, *extra_flags, "-c", "-o", obj, os.path.join(CSRC, src)])
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(force=True, extra_flags=sys.argv[1:]))
