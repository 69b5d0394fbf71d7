"""Compile the C oracle into oracle/libmbulyan_oracle.so with gcc.

Plain -O2, no fast-math, no FMA contraction: the arithmetic stays the one
written in the source.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "mbulyan_oracle.c")
LIB = os.path.join(HERE, "libmbulyan_oracle.so")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math",
           "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


def ensure_built() -> str:
    if (not os.path.exists(LIB)
            or os.path.getmtime(LIB) < os.path.getmtime(SRC)):
        build()
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
