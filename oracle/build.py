"""Compile the CPU oracle (plain C, gcc) into oracle/libsr_oracle.so.

TEST INFRASTRUCTURE: the oracle is the checker, never part of the product
path.  The flags fix the arithmetic contract stated in sr_oracle.c: no FMA
contraction, no fast-math, scalar SSE float evaluation (the x86-64 default).
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sr_oracle.c")
LIB = os.path.join(HERE, "libsr_oracle.so")

CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
          "-fopenmp", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", *CFLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
