"""Compile oracle/givens_oracle.c into oracle/libgivens_oracle.so with gcc.

Building the checker is not using it: the product path never loads this library.
No -ffast-math, so the compiler keeps the source's order of floating-point operations.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "givens_oracle.c")
LIB = os.path.join(HERE, "libgivens_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-ftree-vectorize", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
