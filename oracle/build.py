"""Compile the CPU oracle (plain C, gcc + OpenMP) into two shared libraries:
double precision and, for the extended-precision spot check, long double."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "sinkhorn_oracle.c")
LIB = os.path.join(HERE, "libfs_oracle.so")
LIB_LD = os.path.join(HERE, "libfs_oracle_ld.so")

# No -ffast-math / -Ofast: the oracle keeps IEEE semantics and the written order.
_FLAGS = ["-O2", "-fPIC", "-shared", "-fopenmp", "-std=c11", "-Wall", "-Wextra"]


def _stale(lib: str) -> bool:
    return (not os.path.exists(lib)) or os.path.getmtime(lib) < os.path.getmtime(SRC)


def build(force: bool = False) -> None:
    for lib, extra in ((LIB, []), (LIB_LD, ["-DFSO_LONG_DOUBLE"])):
        if force or _stale(lib):
            subprocess.check_call(["gcc", *_FLAGS, *extra, SRC, "-o", lib, "-lm"])


if __name__ == "__main__":
    build(force=True)
    print("built", LIB, LIB_LD)
