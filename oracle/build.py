"""Compiles the C oracle into oracle/libdsla_oracle.so with gcc.

Test infrastructure only.  Plain -O2, OpenMP over (batch, head) pairs, no
intrinsics, no fast-math: the oracle is meant to be obviously correct, not fast.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "dsla_oracle.c")
LIB = os.path.join(HERE, "libdsla_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
