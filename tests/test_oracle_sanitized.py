"""The CPU checker's pins once more, against a build of the same C source under
AddressSanitizer and UndefinedBehaviorSanitizer (host code only): an access past
a buffer, a misaligned or overflowing index computation or a shift out of range
in the checker aborts the child process."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _asan_runtime():
    try:
        p = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, timeout=30).stdout.strip()
    except Exception:
        return None
    return p if os.path.isabs(p) and os.path.exists(p) else None


def test_checker_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    asan = _asan_runtime()
    if asan is None:
        pytest.skip("gcc's libasan.so is not present in this container")
    from oracle import build as ob_build
    try:
        lib = ob_build.build_sanitized()
    except subprocess.CalledProcessError as e:
        pytest.skip(f"the sanitizer build of the checker does not link here: {e}")
    files = sorted(f for f in glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py"))
                   if not f.endswith("test_oracle_sanitized.py"))
    assert len(files) >= 6
    env = dict(os.environ)
    env["GF_ORACLE_LIB"] = lib
    # the sanitizer runtime has to be the first library of the process; anything already preloaded stays
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter and the numeric libraries are not built for the sanitizer: no leak report at
    # exit, no complaints about their allocator pairing; errors in the checker still abort
    env["ASAN_OPTIONS"] = "detect_leaks=0:alloc_dealloc_mismatch=0:new_delete_type_mismatch=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + files,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert " passed" in r.stdout
    # and the child really ran on the instrumented build
    r = subprocess.run([sys.executable, "-c", "from oracle import binding as b; print(b._lib._name)"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip() == lib, (r.stdout, r.stderr[-2000:])
