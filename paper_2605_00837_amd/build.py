"""Build the C-ABI HIP library for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfastsinkhorn.so")
OBJDIR = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed fp32 VALU forms are switched off for every device compile; matrix-core accumulators stay in
# ordinary vector registers (no copies to and from the accumulation registers around every tile)
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-mllvm", "-amdgpu-mfma-vgpr-form"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _deps_mtime():
    files = sources() + glob.glob(os.path.join(CSRC, "*.h")) + \
        [os.path.join(os.path.dirname(HERE), "include", "fastsinkhorn.h")]
    return max(os.path.getmtime(f) for f in files)


def is_stale() -> bool:
    return (not os.path.exists(LIB)) or os.path.getmtime(LIB) < _deps_mtime()


def build(force: bool = True, verbose: bool = False, extra=()):
    """Compile every .hip source and link libfastsinkhorn.so in-tree."""
    if not force and not is_stale():
        return LIB
    os.makedirs(OBJDIR, exist_ok=True)
    procs = []
    objs = []
    for src in sources():
        obj = os.path.join(OBJDIR, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [HIPCC, *FLAGS, *extra, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines()
                        if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
        if p.returncode != 0:
            failed = True
            print(f"--- {src} FAILED\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(f"--- {src}\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB])
    return LIB


SAN_DIR = os.path.join(OBJDIR, "host_san")
SAN_DRIVER = os.path.join(os.path.dirname(HERE), "tests", "host", "host_sanitize_check.cpp")
SAN_EXE = os.path.join(SAN_DIR, "host_sanitize_check")
# sanitizers on the HOST pass only (each -fsanitize= directly behind -Xarch_host); device code is built as always
_HOST_SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]


def build_host_sanitized(force: bool = False) -> str:
    """The library's sources with their host code under AddressSanitizer + UBSan, linked with the driver
    tests/host/host_sanitize_check.cpp into one executable (CPU only: it never touches a device)."""
    newest = max(_deps_mtime(), os.path.getmtime(SAN_DRIVER))
    if not force and os.path.exists(SAN_EXE) and os.path.getmtime(SAN_EXE) >= newest:
        return SAN_EXE
    os.makedirs(SAN_DIR, exist_ok=True)
    flags = ["-O1", "-g"] + [f for f in FLAGS if f != "-O3"] + _HOST_SAN
    procs, objs = [], []
    for src in sources() + [SAN_DRIVER]:
        obj = os.path.join(SAN_DIR, os.path.basename(src) + ".o")
        objs.append(obj)
        procs.append((src, subprocess.Popen([HIPCC, *flags, "-x", "hip", "-c", src, "-o", obj],
                                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            print(f"--- {src} FAILED\n{out}", file=sys.stderr)
            raise RuntimeError("hipcc failed (host sanitizer build)")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", *_HOST_SAN, *objs, "-o", SAN_EXE])
    return SAN_EXE


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
    if "--host-sanitize" in sys.argv:
        print(build_host_sanitized(force=True))
