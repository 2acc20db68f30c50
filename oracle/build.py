"""Compile the CPU oracle (plain C, gcc + OpenMP) into two shared libraries:
double precision and, for the extended-precision spot check, long double.

`python oracle/build.py --sanitize` (or `build_sanitized()`) builds the sanitizer leg, CPU only: the oracle
with its driver `sanitize_check.c` as one executable under -fsanitize=address,undefined, and a shared library
under -fsanitize=undefined alone that Python can load in place of the ordinary one (the pins then run against
it; `FS_ORACLE_LIB` names the library the front-end loads)."""
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


SAN_DRIVER_SRC = os.path.join(HERE, "sanitize_check.c")
SAN_EXE = os.path.join(HERE, "fs_oracle_san_check")
LIB_UBSAN = os.path.join(HERE, "libfs_oracle_ubsan.so")
_SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-fno-sanitize-recover=all"]


def build_sanitized(force: bool = False):
    """Returns (driver executable, UBSan shared library)."""
    newest = max(os.path.getmtime(SRC), os.path.getmtime(SAN_DRIVER_SRC))
    if force or not os.path.exists(SAN_EXE) or os.path.getmtime(SAN_EXE) < newest:
        subprocess.check_call(["gcc", *_SAN, "-fsanitize=address,undefined", SRC, SAN_DRIVER_SRC, "-o", SAN_EXE, "-lm"])
    if force or not os.path.exists(LIB_UBSAN) or os.path.getmtime(LIB_UBSAN) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", *_SAN, "-fPIC", "-shared", "-fsanitize=undefined", SRC, "-o", LIB_UBSAN, "-lm"])
    return SAN_EXE, LIB_UBSAN


if __name__ == "__main__":
    import sys
    build(force=True)
    print("built", LIB, LIB_LD)
    if "--sanitize" in sys.argv:
        print("built", *build_sanitized(force=True))
