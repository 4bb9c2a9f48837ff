"""Compile the CPU oracle (plain C, gcc) into oracle/libocn_oracle.so.

Test infrastructure only.  Floating-point contraction and fast-math stay off so that each
operation in the oracle rounds exactly once in its own type.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libocn_oracle.so")
SRC = os.path.join(HERE, "ocn_oracle.c")
HDR = os.path.join(HERE, "ocn_oracle.h")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(SRC), os.path.getmtime(HDR)):
        return LIB
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-frounding-math", "-Wall", "-Wextra", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build())
