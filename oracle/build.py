"""Compile the oracle's C file with gcc into oracle/libkvmig_oracle.so."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "kvmig_oracle.c")
LIB = os.path.join(HERE, "libkvmig_oracle.so")


def build(force: bool = False) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC",
                               SRC, "-o", LIB])
    return LIB


if __name__ == "__main__":
    print(build(force=True))
