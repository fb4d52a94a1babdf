"""Compile the CPU oracle (plain C, gcc) into oracle/libulsnn_oracle.so.  Test infrastructure only."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libulsnn_oracle.so")
SOURCES = ["ref_sgemm.c", "ref_mlp.c"]
DEPS = SOURCES + ["ref_mlp_body.inc"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(HERE, s)) > t for s in DEPS)


def build(force: bool = False) -> str:
    if force or stale():
        # -O2 without -ffast-math: sums stay in the index order the source states
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra", "-o", LIB]
        cmd += [os.path.join(HERE, s) for s in SOURCES] + ["-lm"]
        subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
