"""Compile the C oracle with gcc.  Test infrastructure only (see ttkv_oracle.c)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ttkv_oracle.c")
LIB = os.path.join(HERE, "libttkv_oracle.so")


def build(force: bool = True) -> str:
    """gcc -O2, no fast-math, no FMA contraction: every fp32 step of the
    quantizers stays one IEEE operation."""
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
