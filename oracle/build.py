"""Compile the C oracle into oracle/liboracle.so (gcc, -O2, OpenMP over independent outputs).

Building the checker is not using it: the product path never loads this library.
Run as `python oracle/build.py`; also called by __graft_entry__.build().
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "qless_oracle.c")
OUT = os.path.join(HERE, "liboracle.so")


def build(verbose=True):
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-fPIC", "-shared", "-Wall", "-Wno-misleading-indentation", "-Wno-unknown-pragmas",
           SRC, "-o", OUT, "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return OUT


if __name__ == "__main__":
    build()
    sys.exit(0)
