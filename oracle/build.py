"""Compiles the CPU oracle (test infrastructure) into oracle/libfloe_oracle.so with g++."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libfloe_oracle.so")
SRC = [os.path.join(HERE, "floe_oracle.cpp")]
HDR = [os.path.join(HERE, "floe_oracle.h")]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SRC + HDR)


def build(force: bool = False) -> str:
    if force or stale():
        cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
               "-pthread", "-Wall", "-Wextra", "-o", LIB] + SRC
        subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
