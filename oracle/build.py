"""Compile the CPU oracle (plain C) into oracle/liblutnn_oracle.so.

Test infrastructure only; see the header of lutnn_oracle.c.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "lutnn_oracle.c")
LIB = os.path.join(HERE, "liblutnn_oracle.so")

# -ffp-contract=off: the only fused operations are the explicit fmaf() calls.
CMD = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fvisibility=hidden", "-shared", "-fPIC",
       "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    subprocess.run(CMD, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
