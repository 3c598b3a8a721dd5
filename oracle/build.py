"""Compile the oracle's C source into oracle/libfforacle.so with gcc.

Test infrastructure: the HIP library does not depend on this file or its output.
-ffp-contract=off keeps one rounding per written fp32 operation (gcc would
otherwise fuse a*b+c on machines with FMA)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ff_oracle.c")
LIB = os.path.join(HERE, "libfforacle.so")


def build(force: bool = False) -> str:
    if (not force) and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-fPIC", "-shared", "-std=c11",
           "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
           "-o", LIB + ".tmp", SRC, "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
