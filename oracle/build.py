"""Compile the C oracle into oracle/libref_stream.so (gcc, OpenMP, no fast-math).

Building the checker is not using it: the product never loads this library.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ref_stream.c")
LIB = os.path.join(HERE, "libref_stream.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    # Generic x86-64 code on purpose: the library is built on one machine and
    # run on another.  No -ffast-math: summation order stays as written.
    cmd = ["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
    sys.exit(0)
