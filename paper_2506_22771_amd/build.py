"""Build libffint8.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2506_22771_amd.build [--force]

-ffp-contract=off: the numerics need one rounding per written fp32 operation (hipcc would fuse).
-packed-fp32-ops is switched off as required on the test machines."""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libffint8.so")
SOURCES = ["elementwise.hip", "gemm_i8.hip", "conv.hip", "fused.hip", "api.hip"]
HEADERS = [os.path.join(CSRC, "ff_internal.hpp"), os.path.join(CSRC, "device_math.hpp"), os.path.join(os.path.dirname(HERE), "include", "ffint8.h")]
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function", "-Wno-inline-asm"]


def _stale(target: str, deps) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if force or _stale(obj, [path] + HEADERS):
        subprocess.run(["hipcc", *FLAGS, "-c", path, "-o", obj], check=True)
    return obj


def build(force: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or _stale(LIB, objs):
        subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp", *objs], check=True)
        os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
