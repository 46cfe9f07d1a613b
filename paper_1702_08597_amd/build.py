"""Compile libswconv.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libswconv.so")
SOURCES = [os.path.join(CSRC, "swconv.hip")]
HEADERS = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hpp", ".inc"))]
HEADERS.append(os.path.join(os.path.dirname(HERE), "include", "swconv.h"))

# -packed-fp32-ops: keep hipcc from forming packed fp32 VALU instructions (the host pass prints a
# harmless "not a recognized feature" warning for it).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build_library(force: bool = True) -> str:
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        tmp = LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call([hipcc] + HIPCC_FLAGS + ["-o", tmp] + SOURCES)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library())
