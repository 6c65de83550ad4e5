"""Builds the CPU oracle (oracle/libecco_oracle.so) with g++.  Test infrastructure only."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libecco_oracle.so")
SRCS = [os.path.join(HERE, n) for n in ("ecco_oracle.cpp", "ecco_paper_block.cpp")]
HDRS = [os.path.join(HERE, n) for n in ("ecco_oracle.h", "ecco_paper_block.h")]


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(f) for f in SRCS + HDRS):
        return LIB
    cmd = ["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-Wall", "-Wextra",
           "-shared", "-fPIC", *SRCS, "-o", LIB]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
