"""Compile the oracle's C translation unit with gcc (test infrastructure only).

Usage: ``python -m oracle.build``.  Produces ``oracle/libcf_oracle.so``.
Plain ``-O2 -fopenmp``: the oracle is never tuned.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cf_oracle.c")
LIB = os.path.join(HERE, "libcf_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
