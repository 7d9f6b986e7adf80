"""Compile the oracle's C file into oracle/libfact_oracle.so with gcc.

Test infrastructure: building the checker is not using it.  No fast-math flag
is given, so every sum keeps the order written in the source.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fact_oracle.c")
LIB = os.path.join(HERE, "libfact_oracle.so")


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-std=c11", "-O3", "-mavx2", "-mfma", "-fopenmp", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
