"""Compile the C oracle (``rsr_oracle.c``) into ``librsr_oracle.so`` with gcc.

Test infrastructure: called by the package build step and, on demand, by
``oracle.dense`` when the shared object is missing or older than its source.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "rsr_oracle.c")
LIB = os.path.join(HERE, "librsr_oracle.so")


def build(force: bool = False) -> str:
    stale = (not os.path.exists(LIB)) or os.path.getmtime(LIB) < os.path.getmtime(SRC)
    if force or stale:
        tmp = LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra", "-o", tmp, SRC]
        subprocess.run(cmd, check=True)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
