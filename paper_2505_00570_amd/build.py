"""Build libfreqkv.so (gfx950) in-tree with hipcc.  `python -m paper_2505_00570_amd.build`."""
from __future__ import annotations

import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB_DIR = os.path.join(PKG, "lib")
OBJ_DIR = os.path.join(PKG, "_build")
LIB = os.path.join(LIB_DIR, "libfreqkv.so")
SOURCES = ["freqkv_kernels.hip", "freqkv_fast.hip", "freqkv_attend.hip", "freqkv_prefill.hip", "freqkv_api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops off: the device compiler must not form v_pk_{add,mul,fma}_f32 from float code.  The
# flag reaches both passes of hipcc: the gfx950 pass honours it, the x86 host pass prints "not a recognized
# feature for this target (ignoring feature)", once per file, which is harmless.  The build does not rely on
# that: it keeps the device assembly of every file (-save-temps) and fails if a packed fp32 instruction is
# in it (check_device_asm).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-save-temps=obj",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
PACKED_FP32 = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")


M0_USE = re.compile(r"\bm0\b")
M0_OWN = re.compile(r"^\s*s_mov_b32 m0, s\d+\s*$")


def check_device_asm(asm_path: str) -> tuple:
    """(packed fp32 arithmetic instructions, uses of M0 other than the LDS-address move of the
    global -> LDS copies) in a device assembly file; both must be zero.  The compiler refuses M0 in an
    inline-assembly clobber list (a reserved register), so that M0 has no user besides those copies is
    checked here, on the code it produced."""
    packed = foreign_m0 = 0
    with open(asm_path, "r", errors="replace") as f:
        for line in f:
            code = line.split(";", 1)[0]
            if PACKED_FP32.search(code):
                packed += 1
            if M0_USE.search(code) and not M0_OWN.match(code):
                foreign_m0 += 1
    return packed, foreign_m0


def build(verbose: bool = True) -> str:
    os.makedirs(LIB_DIR, exist_ok=True)
    os.makedirs(OBJ_DIR, exist_ok=True)
    def compile_one(src: str) -> str:
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        asm = os.path.join(OBJ_DIR, src.replace(".hip", "-hip-amdgcn-amd-amdhsa-gfx950.s"))
        packed, foreign_m0 = check_device_asm(asm)
        if packed or foreign_m0:
            raise RuntimeError("%s: %d packed fp32 instructions, %d foreign uses of M0 in the device code"
                               % (src, packed, foreign_m0))
        return obj

    # the files are independent: compile them side by side (hipcc itself is single-threaded per file)
    with ThreadPoolExecutor(max_workers=min(4, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
