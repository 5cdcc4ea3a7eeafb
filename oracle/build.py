"""Compile the C part of the oracle (conv_fp64.c) into oracle/liboracle_conv.so with gcc + OpenMP.

TEST INFRASTRUCTURE ONLY (see conv_fp64.c).  Usage: python -m oracle.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "conv_fp64.c")
LIB = os.path.join(HERE, "liboracle_conv.so")


def build(force: bool = True) -> str:
    """Build the shared object; with force=False an up-to-date one is kept."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
