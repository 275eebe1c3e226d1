"""Compile the fp64 CPU oracle (test infrastructure) into oracle/libvla_oracle.so.

Generic x86-64 code only (no -march=native): the shared object is built on one
machine and loaded on another.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "vla_oracle.c")
OUT = os.path.join(HERE, "libvla_oracle.so")


def build(verbose: bool = False) -> str:
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
           "-ffp-contract=off", SRC, "-o", OUT, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
