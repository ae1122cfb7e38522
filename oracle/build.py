"""Compile oracle/w4a16_oracle.c into oracle/libw4a16_oracle.so with gcc.

Plain C, -O2, no fast-math, no FMA contraction (the fp32 accumulation mode must round
every product and every addition separately), OpenMP for the timed multi-core run.
"""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
SRC = HERE / "w4a16_oracle.c"
LIB = HERE / "libw4a16_oracle.so"


def build(verbose: bool = False) -> pathlib.Path:
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", str(LIB), str(SRC)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
