"""Build step: every HIP source under csrc/ compiled for gfx950 with hipcc and linked into
libshiftattn.so next to this file (in-tree, so it travels with the repo); the benchmark's
reference kernels under bench_kernels/ go into a shared object of their own, libspceilings.so.

``python -m paper_2507_11830_amd.build --sanitize-host`` builds a second copy of libshiftattn
whose HOST code is instrumented with AddressSanitizer + UndefinedBehaviorSanitizer
(_build/san/libshiftattn_san.so; device code is unchanged) for the CPU-only boundary tests."""
from __future__ import annotations

import glob
import os
import re
import shlex
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ_DIR = os.path.join(HERE, "_build")
BENCH_SRC = os.path.join(HERE, "bench_kernels")
LIB = os.path.join(HERE, "libshiftattn.so")
CEIL_LIB = os.path.join(HERE, "libspceilings.so")
SAN_LIB = os.path.join(OBJ_DIR, "san", "libshiftattn_san.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    *shlex.split(os.environ.get("SP_HIPCC_EXTRA", "")),   # extra compiler flags for experiments
]
# host-side instrumentation only: each -fsanitize= goes directly behind -Xarch_host
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


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


def loop_spills(asm: str) -> dict:
    """Scratch (register spill) instructions inside loops, per kernel of an assembly listing.
    The prefill kernel sits at the register limit, and where the allocator puts its spill code
    changes with unrelated edits; a reload on the tile loop's common path costs 5-20 % (it is
    waited for right before the period's barrier).  Loop membership comes from the compiler's
    own block comments ("in Loop: Header=...")."""
    out, kern, inloop = {}, None, False
    with open(asm) as f:
        lines = f.read().split("\n")
    i = 0
    while i < len(lines):
        line = lines[i]
        m = re.match(r"^(_Z\w+):", line)
        if m:
            kern, inloop = m.group(1), False
            out[kern] = 0
        elif line.startswith(".Lfunc_end"):
            kern = None
        elif kern and (line.startswith(".LBB") or line.strip().startswith("; %bb.")):
            text, j = line, i + 1
            while j < len(lines) and lines[j].strip().startswith(";") and not lines[j].strip().startswith("; %bb."):
                text += lines[j]
                j += 1
            marked = "in Loop" in text or "Loop Header" in text
            inloop = marked if line.startswith(".LBB") else (inloop or marked)  # fall-through blocks stay in their loop
            i = j
            continue
        elif kern and inloop and "scratch_" in line.split(";")[0]:
            out[kern] += 1
        i += 1
    return out


def _check_loop_spills(src: str, asm: str) -> None:
    """The one-workgroup-per-query-tile prefill kernels (the C5a path) must keep their loops free of
    spill code; the split forms are allowed the few reloads of their rarely taken short-row copy."""
    for kern, n in loop_spills(asm).items():
        if "prefill_kernel" not in kern:
            continue
        main_form = re.search(r"ELb0ELb0E", kern) is not None
        if n > (0 if main_form else 8):
            raise RuntimeError(f"{os.path.basename(src)}: {n} spill instructions inside the loops of {kern}; "
                               "the register allocation moved, look at the listing")


def _compile(src: str, obj_dir: str = OBJ_DIR, extra_flags=(), product: bool = True) -> str:
    base = os.path.basename(src).replace(".hip", "")
    obj = os.path.join(obj_dir, base + ".o")
    with open(src) as f:
        uses_lds_dma = "global_load_lds" in f.read()
    extra = ["-save-temps=obj"] if uses_lds_dma else []
    r = subprocess.run([HIPCC, *FLAGS, *extra_flags, *extra, "-c", src, "-o", obj], capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    if uses_lds_dma:
        asm = os.path.join(obj_dir, base + "-hip-amdgcn-amd-amdhsa-gfx950.s")
        if not os.path.exists(asm):
            raise RuntimeError(f"{os.path.basename(src)}: the compiler left no {asm}; the M0 check cannot run, "
                               "so the build is refused")
        _check_m0(src, asm)
        if product and not os.environ.get("SP_HIPCC_EXTRA"):  # measurement and sanitizer builds may spill
            _check_loop_spills(src, asm)
    return obj


def _link(objs, lib: str, extra_flags=()) -> None:
    tmp = lib + f".tmp{os.getpid()}"
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *extra_flags, "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError(f"link of {lib} failed")
    os.replace(tmp, lib)


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    bench = sorted(glob.glob(os.path.join(BENCH_SRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs) + len(bench))) as ex:
        objs = list(ex.map(_compile, srcs + bench))
    _link(objs[:len(srcs)], LIB)
    _link(objs[len(srcs):], CEIL_LIB)
    if verbose:
        print("built", LIB)
        print("built", CEIL_LIB)
    return LIB


def build_sanitized(verbose: bool = False) -> str:
    """libshiftattn with ASan + UBSan on the host side (argument validation, launch set-up)."""
    out_dir = os.path.dirname(SAN_LIB)
    os.makedirs(out_dir, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda s_: _compile(s_, out_dir, SAN_FLAGS, product=False), srcs))
    _link(objs, SAN_LIB, ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"])
    if verbose:
        print("built", SAN_LIB)
    return SAN_LIB


if __name__ == "__main__":
    if "--sanitize-host" in sys.argv:
        build_sanitized(verbose=True)
    else:
        build(verbose=True)
