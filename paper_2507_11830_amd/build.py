"""Build step for libshiftattn.so: every HIP source under csrc/ compiled for gfx950 with hipcc
and linked into one shared library next to this file (in-tree, so it travels with the repo)."""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libshiftattn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _check_m0(src: str, asm: str) -> None:
    """The direct global->LDS loads are emitted as inline assembly that sets M0 itself; the
    compiler is not told (M0 is a reserved register and cannot be declared clobbered).  That is
    only sound while the compiler uses M0 for nothing in those kernels, so the generated
    assembly is checked: every mention of m0 must be one of our own `s_mov_b32 m0, sN`."""
    bad = []
    with open(asm) as f:
        for n, line in enumerate(f, 1):
            code = line.split(";")[0]
            if "movrel" in code or "s_sendmsg" in code:   # read M0 without naming it
                bad.append(f"{asm}:{n}: {line.rstrip()}")
            elif "m0" in code.split() or " m0," in code or code.rstrip().endswith(" m0"):
                if not re.match(r"^\s*s_mov_b32 m0, s\d+\s*$", code):
                    bad.append(f"{asm}:{n}: {line.rstrip()}")
    if bad:
        raise RuntimeError(f"{os.path.basename(src)}: the compiler uses M0 next to the inline-assembly LDS loads:\n"
                           + "\n".join(bad[:10]))


def _compile(src: str) -> str:
    base = os.path.basename(src).replace(".hip", "")
    obj = os.path.join(OBJ_DIR, base + ".o")
    with open(src) as f:
        uses_lds_dma = "global_load_lds" in f.read()
    extra = ["-save-temps=obj"] if uses_lds_dma else []
    r = subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    if uses_lds_dma:
        _check_m0(src, os.path.join(OBJ_DIR, base + "-hip-amdgcn-amd-amdhsa-gfx950.s"))
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    tmp = LIB + f".tmp{os.getpid()}"
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
