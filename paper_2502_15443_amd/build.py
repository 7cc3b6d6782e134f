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
           os.path.join(PKG, "csrc", "dc_encode.hip"), os.path.join(PKG, "csrc", "dc_probe.hip")]
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


# Vector-ALU instructions a SIMD issues every two cycles for a wavefront (bench.py --issue-rates measures them);
# all others met in the kernels take four.
TWO_CYCLE = {"v_and_b32", "v_or_b32", "v_xor_b32", "v_add_u32", "v_sub_u32", "v_subrev_u32", "v_lshrrev_b32", "v_mov_b32",
             "v_mul_f32", "v_add_f32", "v_cndmask_b32", "v_lshrrev_b16", "v_add_u16"}


def loop_mix(asm_text: str) -> dict:
    """Vector-ALU instructions of the main loop (the innermost loop with the most table look-ups) of every decode
    kernel at 256 sub-streams, Huffman, by issue class: {mode: {"valu": n, "two_cycle": a, "four_cycle": b,
    "cycles_per_instruction": c, "lookups": symbols a turn}}."""
    out = {}
    for mode, label in ((0, "int8"), (1, "bf16"), (2, "gemv")):
        m = re.search(r"^(_ZN\S*dc_decode_kernelILi256ELi%dELi0ELb0E\S*):" % mode, asm_text, re.M)
        if not m:
            continue
        body = asm_text[m.start():asm_text.index(".Lfunc_end", m.start())].split("\n")
        at = {mm.group(1): i for i, ln in enumerate(body) for mm in [re.match(r"(\.LBB\d+_\d+):", ln)] if mm}
        best = None
        for i, ln in enumerate(body):
            mm = re.search(r"s_c?branch\w*\s+(\.LBB\d+_\d+)", ln)
            if mm and mm.group(1) in at and at[mm.group(1)] < i:
                a, b = at[mm.group(1)], i
                n = sum("ds_read_u16" in x for x in body[a:b])
                if best is None or n > best[0] or (n == best[0] and b - a < best[2] - best[1]):
                    best = (n, a, b)
        n, a, b = best
        two = four = 0
        for ln in body[a:b + 1]:
            mm = re.match(r"\s*(v_\w+)", ln)
            if not mm:
                continue
            name = mm.group(1)
            plain = not name.endswith(("_sdwa", "_dpp", "_e64"))
            if plain and re.sub(r"_e32$", "", name) in TWO_CYCLE:
                two += 1
            else:
                four += 1
        out[label] = {"valu": two + four, "two_cycle": two, "four_cycle": four,
                      "cycles_per_instruction": round((2 * two + 4 * four) / (two + four), 3), "lookups": n}
    return out


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + HEADERS + [os.path.abspath(__file__)])


def build(force: bool = True, extra=(), want_mix: bool = False) -> str:
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
                text = f.read()
            hit = PACKED_FP32.search(text)
            if hit:
                raise RuntimeError(f"packed fp32 operation {hit.group(0)} in {os.path.basename(path)}")
            if want_mix and "dc_decode_kernel" in text:
                import json
                print(json.dumps({"main_loop_instruction_mix": loop_mix(text)}))
        shutil.move(out, LIB)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    # --loop-mix: also print the instruction mix of the decode kernels' main loops (one JSON line)
    args = [a for a in sys.argv[1:] if a != "--loop-mix"]
    print(build(True, args, want_mix="--loop-mix" in sys.argv[1:]))
