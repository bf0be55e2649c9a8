"""Compile the CPU oracle (test infrastructure) into oracle/libslicer_ref.so."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "slicer_ref.c")
LIB = os.path.join(HERE, "libslicer_ref.so")

# -ffp-contract=off / -fno-fast-math: every fp32 operation is one IEEE RNE operation.
FLAGS = ["-O2", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off", "-fno-fast-math",
         "-fopenmp", "-shared", "-fPIC"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "slicer_ref.h"))):
        return LIB
    subprocess.run(["gcc", *FLAGS, SRC, "-o", LIB, "-lm"], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
