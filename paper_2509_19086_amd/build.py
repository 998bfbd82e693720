"""Builds libsja.so (the C-ABI library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libsja.so")
SOURCES = [os.path.join(CSRC, "sja.hip")]


def headers() -> list:
    """Every header the library is built from: all of csrc/ plus the public one."""
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")) + \
        [os.path.join(os.path.dirname(_HERE), "include", "sja.h")]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def command() -> list:
    # amdgpu-kernarg-preload-count: the first 16 dwords of a kernel's arguments arrive in scalar
    # registers with the wave instead of being loaded by it (gfx940 and later; the compiler keeps
    # a loading prologue for firmware that does not preload).  A resolve round is one short kernel
    # whose first memory trip otherwise waits for that load; the round kernel's argument order
    # puts what that trip needs first.
    return [hipcc(), "-O3", "-std=c++17", "--offload-arch=gfx950", "-shared", "-fPIC",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-mllvm", "-amdgpu-kernarg-preload-count=16",
            "-Wall", "-Wno-unused-function",
            "-o", LIB] + SOURCES


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + headers())


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library; force=False skips the compile when it is up to date."""
    if force or is_stale():
        cmd = command()
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print(LIB)
