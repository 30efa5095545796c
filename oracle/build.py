"""Compile the C part of the oracle (test infrastructure) with gcc.

Portable flags only: the shared object is built on one machine and may be
loaded on another, so no -march=native, and no FMA contraction so that a sum
is the same sequence of roundings wherever it runs.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rtp_oracle.c")
LIB = os.path.join(HERE, "librtp_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O3", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
