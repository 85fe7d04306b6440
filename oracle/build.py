"""Compile the float64 CPU oracle (plain C, gcc) into oracle/libesrnn_oracle.so.

Test infrastructure only; the HIP library never links or loads this.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "esrnn_oracle.c")
HDR = os.path.join(HERE, "esrnn_oracle.h")
LIB = os.path.join(HERE, "libesrnn_oracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(SRC), os.path.getmtime(HDR))
        if os.path.getmtime(LIB) >= newest:
            return LIB
    cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
