"""CPU-only sanitizer leg: the fp64 oracle and the HOST side of the C-ABI library (argument
validation, launch set-up, error reporting) rebuilt with AddressSanitizer +
UndefinedBehaviorSanitizer, and the pin tests resp. the no-GPU boundary tests re-run on those
builds in a child process that has the matching sanitizer runtime preloaded.  Device code is
never instrumented and nothing here touches a GPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _preload(runtime: str) -> str:
    """The sanitizer runtime has to come first; whatever is preloaded already stays behind it."""
    old = os.environ.get("LD_PRELOAD", "")
    return runtime + (":" + old if old else "")


def _run(env_extra, args):
    env = dict(os.environ)
    env.update(env_extra)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"   # the interpreter's own allocations are not ours to judge
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *args], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    return r.stdout


def test_oracle_pins_under_asan_ubsan():
    rt = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("gcc's libasan is not installed")
    out = _run({"SP_ORACLE_SANITIZE": "1", "LD_PRELOAD": _preload(rt)}, ["tests/test_oracle_pins.py"])
    assert " passed" in out


def test_boundary_host_code_under_asan_ubsan():
    from paper_2507_11830_amd import build as b

    rt = subprocess.check_output([os.path.join(os.path.dirname(b.HIPCC), "..", "llvm", "bin", "clang"),
                                  "--print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    if not os.path.isabs(rt) or not os.path.exists(rt):
        pytest.skip("clang's ASan runtime is not installed")
    b.build_sanitized()
    out = _run({"SP_LIB_SANITIZE": "1", "LD_PRELOAD": _preload(rt)},
               ["tests/test_boundary.py", "-k",
                "argument_validation or tuning_keys or workspace_size or hint_validation or per_thread or status_strings"])
    assert " passed" in out
