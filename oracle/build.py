"""Compile the CPU oracle (plain C, fp64, OpenMP) into oracle/libturborag_oracle.so.

Test infrastructure: only the tests, the smoke check and the bench's
cpu_baseline leg build or load this library.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "turborag_oracle.c")
LIB = os.path.join(HERE, "libturborag_oracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    # -O2 without -ffast-math: keep IEEE double semantics and the written summation order.
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
