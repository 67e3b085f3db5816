"""Compile the CPU oracle (plain C, gcc, OpenMP) into oracle/libpq_oracle.so.

The oracle is test infrastructure; building it is not using it.  Contraction of
a*b+c into a fused multiply-add is switched off so that the encode distances are
the same IEEE double operations on every machine.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "pq_oracle.c")
SRC16 = os.path.join(HERE, "pq_oracle16.c")
LIB = os.path.join(HERE, "libpq_oracle.so")


def build(force: bool = False) -> str:
    if (not force) and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(SRC), os.path.getmtime(SRC16)):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", LIB, SRC, SRC16, "-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
