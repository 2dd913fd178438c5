"""Compile the C part of the CPU oracle (test infrastructure) into oracle/liborc.so.

Usage: python oracle/build_oracle.py
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "jz_oracle.c")
OUT = os.path.join(HERE, "liborc.so")


def build(verbose: bool = False) -> str:
    # No -ffast-math: the sums keep the order the source states.
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", OUT, SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
