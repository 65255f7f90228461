"""Compile the C oracle with gcc (test infrastructure; the product never loads it).

`python -m oracle.build` writes oracle/libgemm_oracle.so.  Plain -O3 without
-ffast-math and without -march flags: the same binary must run on any x86-64
host and may not reassociate the fp64 sums.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "gemm_oracle.c")
LIB = os.path.join(HERE, "libgemm_oracle.so")


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O3", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math", "-Wall", "-Wextra",
           "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
    sys.exit(0)
