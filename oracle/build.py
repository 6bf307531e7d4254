"""Compile the CPU oracle (plain C, gcc) into oracle/libdcnv4_oracle.so.

Test infrastructure: building the checker is not using it.  Run as
`python oracle/build.py` or call `build()`.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dcnv4_oracle.c")
LIB = os.path.join(HERE, "libdcnv4_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
