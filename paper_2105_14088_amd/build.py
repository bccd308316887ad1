"""Compiles the HIP sources under csrc/ into paper_2105_14088_amd/libcc.so for gfx950."""
from __future__ import annotations

import glob
import os
import re
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcc.so")
SOURCES = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
HEADERS = sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + [os.path.join(os.path.dirname(HERE), "include", "cc.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-FP32 instruction selection off (integer-only code, but applies to every HIP translation unit)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


# Operand-reversed VOP2 opcodes in their DPP form: measured on gfx950 with this toolchain,
# "v_subrev_u32_dpp d, a, b <rotate>" yields rotate(b) - a, not b - rotate(a) (the plain and the non-reversed DPP
# forms, v_sub_u32_dpp / v_add_u32_dpp / v_mov_b32_dpp, behave as documented).  The compiler's DPP combiner can
# produce the form by itself from "x - rotate(y)"; a build that contains one is refused, and the source is changed
# so that the rotate stays an instruction of its own (an empty asm statement with the value as in/out operand).
FORBIDDEN_ISA = re.compile(r"^\s*(v_\w*rev\w*_dpp)\b", re.M)


def check_device_isa(folder: str) -> None:
    for path in sorted(glob.glob(os.path.join(folder, "*-hip-amdgcn-amd-amdhsa-gfx950.s"))):
        with open(path) as fh:
            hit = FORBIDDEN_ISA.search(fh.read())
        if hit:
            raise RuntimeError(f"{os.path.basename(path)}: the compiler emitted {hit.group(1)}, which does not "
                               "compute what its operands say on gfx950; keep the rotate out of the subtraction")


def needs_build() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    if force or needs_build():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        # the intermediate files (device assembly among them) go to a scratch folder and are checked before the
        # library is put in place
        with tempfile.TemporaryDirectory(prefix="cc_build_") as tmp:
            out = os.path.join(tmp, "libcc.so")

            def compile_one(src: str) -> str:
                obj = os.path.join(tmp, os.path.basename(src) + ".o")
                cmd = [hipcc] + HIPCC_FLAGS + ["-save-temps", "-c", src, "-o", obj]
                if verbose:
                    print(" ".join(cmd), flush=True)
                subprocess.check_call(cmd, cwd=tmp)
                return obj

            # one translation unit per source, a few at a time
            with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
                objects = list(pool.map(compile_one, SOURCES))
            check_device_isa(tmp)
            link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objects + ["-o", out]
            if verbose:
                print(" ".join(link), flush=True)
            subprocess.check_call(link, cwd=tmp)
            shutil.move(out, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build(force=True, verbose=True))
