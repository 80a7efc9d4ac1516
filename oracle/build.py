"""Compile the CPU oracle (plain C, gcc) into oracle/libqpo.so.  Test infrastructure only."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["qpo.c", "qpo_encode.c", "qpo_kmeans.c"]
LIB = os.path.join(HERE, "libqpo.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB):
        src_m = max(os.path.getmtime(os.path.join(HERE, s)) for s in SOURCES)
        if os.path.getmtime(LIB) >= src_m:
            return LIB
    cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB] + [os.path.join(HERE, s) for s in SOURCES] + ["-lm"]
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
