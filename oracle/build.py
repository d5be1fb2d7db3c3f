"""Compile the CPU oracle (plain C, gcc) into oracle/libkvswap_oracle.so.

TEST INFRASTRUCTURE ONLY: the oracle is the checker, not part of the product.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "kvswap_oracle.c")
LIB = os.path.join(HERE, "libkvswap_oracle.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "kvswap_oracle.h"))):
        return LIB
    # -ffp-contract=off / no -ffast-math: every fp64 operation rounds exactly as written.
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
