"""Compile libsparq.so (HIP, gfx950 only) in-tree with hipcc.  No GPU needed to build.

Every source is compiled to an object of its own (in parallel, objects under _build/) and the objects are
linked into the shared library.  `--stage-clocks` builds a second library, libsparq_clocks.so, whose
one-workgroup-per-head kernel records time stamps per stage (profiling only: bench.py --stage-clocks).
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsparq.so")
LIB_CLOCKS = os.path.join(HERE, "libsparq_clocks.so")
SOURCES = ["api.hip", "sparq_decode.hip", "sparq_decode_split.hip", "sparq_decode_shared.hip", "sparq_decode_shared_split.hip", "sparq_decode_single_k.hip", "sparq_decode_long.hip", "sparq_decode_bucket.hip", "dense_decode.hip", "kv_append.hip"]
HEADERS = ["common.h", "params.h", "decode_stages.h", "group_stages.h", os.path.join("..", "..", "include", "sparq.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = False, verbose: bool = False, stage_clocks: bool = False) -> str:
    lib = LIB_CLOCKS if stage_clocks else LIB
    if not stage_clocks and not force and not stale():
        return lib
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(OBJ, "clocks") if stage_clocks else OBJ
    os.makedirs(obj_dir, exist_ok=True)
    extra = ["-DSPARQ_STAGE_CLOCKS"] if stage_clocks else []

    def compile_one(src: str) -> str:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [hipcc] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True, stage_clocks="--stage-clocks" in sys.argv))
