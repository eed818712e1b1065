"""Compile the C oracle into oracle/libsbi_oracle.so with gcc (no HIP, no GPU).

TEST INFRASTRUCTURE ONLY: nothing on the product path builds or loads this.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sbi_oracle.c")
LIB = os.path.join(HERE, "libsbi_oracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    # -O2, no fast-math: the summation order written in the source is the one executed.
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
