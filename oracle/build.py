"""Compile the CPU oracle (plain C, gcc) into oracle/libsrq_oracle.so.

Test infrastructure only: the product library never links or loads this.
`-ffp-contract=off` matters: the oracle's binary32 steps must each round once.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "srq_oracle.c")
LIB = os.path.join(HERE, "libsrq_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra",
           "-shared", "-fPIC", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
