"""Compile the C oracle into oracle/libpqc_oracle.so (host code only, gcc)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "pqc_oracle.c")
LIB = os.path.join(HERE, "libpqc_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fopenmp-simd", "-ffp-contract=off", "-mavx2", "-mfma",
           "-Wall", "-Wextra", "-shared", "-fPIC", SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
