"""Compile the C oracle into oracle/liboracle.so (gcc, generic x86-64, OpenMP).

Test infrastructure only.  No -march=native: the library built in one container
is also loaded on the GPU machine, whose host CPU may differ.  Floating-point
contraction is off so every product and sum rounds once, in source order.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "aurora_oracle.c"), os.path.join(HERE, "trace_oracle.c")]
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in SRCS):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-shared", "-fPIC"] + SRCS + ["-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
