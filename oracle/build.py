"""Builds liboracle.so from gemm_oracle.c with gcc.  TEST INFRASTRUCTURE ONLY.

-ffp-contract=off keeps every multiply and add separately rounded (no FMA), which is
what makes the FP32 product "naive".  -mavx2 only widens the j loop; it cannot change
any element's operation order.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liboracle.so")
SRC = os.path.join(HERE, "gemm_oracle.c")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-ftree-vectorize", "-mavx2", "-ffp-contract=off", "-fno-fast-math",
           "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra", "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
