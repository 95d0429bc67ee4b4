"""Compile the C oracle into oracle/libcngp_oracle.so with gcc.

Building the checker is not using it: the product library never links or
loads this file.  -ffp-contract=off keeps the single fp32 multiply of the
coordinate scaling a plain IEEE multiply (no fused multiply-add).
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cngp_oracle.c")
LIB = os.path.join(HERE, "libcngp_oracle.so")


def build(force: bool = False) -> str:
    if (not force and os.path.exists(LIB)
            and os.path.getmtime(LIB) >= os.path.getmtime(SRC)):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
           "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
