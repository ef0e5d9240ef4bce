"""Compile the plain-C oracle routines (smat_ref.c) into oracle/libsmat_ref.so with gcc.

TEST INFRASTRUCTURE: building the checker is not using it; nothing in the
product path loads the result.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "smat_ref.c")
OUT = os.path.join(HERE, "libsmat_ref.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(OUT) and os.path.getmtime(OUT) >= os.path.getmtime(SRC):
        return OUT
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", OUT, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build())
