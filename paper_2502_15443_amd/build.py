"""Builds libdc_mi355x.so (host C++ + gfx950 HIP kernels) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import re
import shutil
import subprocess
import sys
import tempfile

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libdc_mi355x.so")
SOURCES = [os.path.join(PKG, "csrc", "dc_host.cpp"), os.path.join(PKG, "csrc", "dc_decode.hip"),
           os.path.join(PKG, "csrc", "dc_encode.hip")]
HEADERS = [os.path.join(ROOT, "include", "dc.h"), os.path.join(PKG, "csrc", "dc_device.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed fp32 VALU forms (v_pk_add_f32, v_pk_mul_f32, v_pk_fma_f32) are kept out of the device code.  The switch
# is a target feature of the device pass; the driver cannot hand a -Xclang pair to one pass only, so the host
# passes see it too and answer that they do not know it: those lines are dropped from what the build prints.
# That the device pass obeyed is checked below on the assembly the compiler leaves behind.
NO_PACKED_FP32 = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    *NO_PACKED_FP32,
    "-I", os.path.join(ROOT, "include"),
]
HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
PACKED_FP32 = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS + [os.path.abspath(__file__)])


def build(force: bool = True, extra=()) -> str:
    if not (force or stale()):
        return LIB
    tmp = tempfile.mkdtemp(prefix="dc_build_")
    try:
        out = os.path.join(tmp, "libdc_mi355x.so")
        cmd = [HIPCC] + FLAGS + ["-save-temps=obj"] + list(extra) + SOURCES + ["-o", out]
        done = subprocess.run(cmd, cwd=tmp, stderr=subprocess.PIPE, text=True)
        noise = [ln for ln in done.stderr.splitlines() if ln.strip() and ln.strip() != HOST_PASS_NOTE]
        if noise:
            print("\n".join(noise), file=sys.stderr)
        if done.returncode != 0:
            raise subprocess.CalledProcessError(done.returncode, cmd)
        device_asm = glob.glob(os.path.join(tmp, "*gfx950*.s"))
        if not device_asm:
            raise RuntimeError("the compiler left no device assembly to check")
        for path in device_asm:
            with open(path) as f:
                hit = PACKED_FP32.search(f.read())
            if hit:
                raise RuntimeError(f"packed fp32 operation {hit.group(0)} in {os.path.basename(path)}")
        shutil.move(out, LIB)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(True, sys.argv[1:]))
