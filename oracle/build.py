"""Compile oracle/moe_oracle.c into oracle/libmoe_oracle.so with gcc (test infrastructure)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "moe_oracle.c")
LIB = os.path.join(HERE, "libmoe_oracle.so")

# x86-64-v3 (AVX2+FMA) rather than -march=native: the library is built on one machine and
# run on another. -ffp-contract=off keeps every fp32 operation exactly as written; the one
# fused multiply-add the definition needs is an explicit fmaf().
CFLAGS = ["-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
          "-Wall", "-Wextra", "-std=c11"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", *CFLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
