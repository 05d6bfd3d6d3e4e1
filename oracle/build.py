"""Compile the reference CPU implementation (test infrastructure) with gcc.

    python -m oracle.build

Produces oracle/libmx_oracle.so next to the sources.  Building the checker is
not using it: the GPU library never links or loads this file.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libmx_oracle.so")
SRC = os.path.join(HERE, "mx_oracle.c")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
        os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "mx_oracle.h"))
    ):
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
