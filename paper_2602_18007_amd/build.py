"""Builds libhxt.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to compile."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libhxt.so")
SOURCES = [os.path.join(PKG, "csrc", "hxt_device.hip"), os.path.join(PKG, "csrc", "hxt_plan.cpp")]
HEADERS = [os.path.join(PKG, "csrc", "hxt_internal.h"), os.path.join(PKG, "csrc", "hxt_kernels.h"),
           os.path.join(ROOT, "include", "hxt.h")]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def command() -> list:
    return [
        hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wextra", "-Wno-unused-parameter",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(PKG, "csrc"),
        "-o", LIB, *SOURCES,
    ]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS)


def build(force: bool = True) -> str:
    if force or stale():
        subprocess.run(command(), check=True)
    return LIB


if __name__ == "__main__":
    print(build())
