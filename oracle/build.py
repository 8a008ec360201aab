"""Build the CPU oracle (test infrastructure) into oracle/libsoar_oracle.so.

Plain gcc, no vector or FMA target flags: fmaf() resolves to the C library's
correctly rounded routine, and -ffp-contract=off keeps every other operation a
separate IEEE binary32 operation.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "soar_oracle.c")
OUT = os.path.join(HERE, "libsoar_oracle.so")
FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
         "-fno-fast-math", "-Wall", "-Wextra"]


def build(verbose: bool = False) -> str:
    cmd = ["gcc", *FLAGS, SRC, "-o", OUT, "-lm"]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return OUT


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
