"""Compile the C oracle (gcc -O2, OpenMP) into oracle/liboob_oracle.so."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oob_oracle.c")
SRCS = [SRC, os.path.join(HERE, "oob_inst_oracle.c"), os.path.join(HERE, "oob_exact_oracle.c")]
LIB = os.path.join(HERE, "liboob_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(x) for x in SRCS):
        return LIB
    cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB] + SRCS
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
