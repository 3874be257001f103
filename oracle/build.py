"""Compile the CPU oracle (plain C, gcc) into oracle/libaride_oracle.so.

Test infrastructure only: nothing in the product package imports this.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "aride_oracle.c")
LIB = os.path.join(HERE, "libaride_oracle.so")


def build(verbose: bool = False) -> str:
    # -ffp-contract=off: the oracle's arithmetic is the written expression, one
    # rounding per operation, with no fused multiply-adds introduced by the compiler.
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
