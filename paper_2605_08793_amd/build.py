"""Compile the HIP library in-tree: paper_2605_08793_amd/libregot.so (gfx950 only)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", "regot.hip"), os.path.join(HERE, "csrc", "regot_pattern.hip")]
LIB = os.path.join(HERE, "libregot.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def build(verbose: bool = False, extra=()) -> str:
    cmd = ["hipcc", *HIPCC_FLAGS, *extra, *SRCS, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
