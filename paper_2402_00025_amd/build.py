"""Compile the HIP sources into paper_2402_00025_amd/libw4a16.so for gfx950 (cross-compiles
without a GPU).  The library is built in-tree so it travels with the source tree."""
from __future__ import annotations

import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
SRC = HERE / "csrc" / "w4a16.hip"
LIB = HERE / "libw4a16.so"

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-munsafe-fp-atomics",                                     # hardware fp32 / packed-fp16 atomic adds
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no v_pk_*_f32
    "-mllvm", "-amdgpu-kernarg-preload-count=14",                # leading kernel arguments arrive in SGPRs
    "-Wall", "-Wno-unused-function",
]


def build(verbose: bool = False, extra=()) -> pathlib.Path:
    cmd = ["hipcc", *HIPCC_FLAGS, *extra, "-o", str(LIB), str(SRC)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
