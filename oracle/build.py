"""Compile the CPU oracle (oracle/qnn_oracle.c) into oracle/liboracle.so with gcc.

Test infrastructure: building the checker is not using it.  Plain -O3 for a generic
x86-64 target (the library travels to other hosts), OpenMP over output rows only,
and -ffp-contract=off so every fp32 step of the quantizer is a single IEEE op.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "qnn_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")


def build(force=True):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O3", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", "-shared", "-fPIC", SRC, "-o", LIB + ".tmp", "-lm"]
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    print(build())
