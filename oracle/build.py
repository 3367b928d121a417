"""Compile the oracle's C file with gcc into oracle/liboracle.so (test infrastructure only)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "fptq_oracle.c")
LIB = os.path.join(HERE, "liboracle.so")

# -ffp-contract=off: the quantizer's single fp32 multiply must not be fused with anything.
CFLAGS = ["-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", *CFLAGS, SRC, "-o", LIB, "-lm"])
    return LIB


if __name__ == "__main__":
    print(build())
