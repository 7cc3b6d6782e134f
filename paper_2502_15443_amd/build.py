"""Builds libdc_mi355x.so (host C++ + gfx950 HIP kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libdc_mi355x.so")
SOURCES = [os.path.join(PKG, "csrc", "dc_host.cpp"), os.path.join(PKG, "csrc", "dc_decode.hip"),
           os.path.join(PKG, "csrc", "dc_encode.hip")]
HEADERS = [os.path.join(ROOT, "include", "dc.h"), os.path.join(PKG, "csrc", "dc_device.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # packed fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"),
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS + [os.path.abspath(__file__)])


def build(force: bool = True, extra=()) -> str:
    if force or stale():
        cmd = [HIPCC] + FLAGS + list(extra) + SOURCES + ["-o", LIB]
        subprocess.check_call(cmd, cwd=PKG)
    return LIB


if __name__ == "__main__":
    print(build(True, sys.argv[1:]))
