"""The oracle's pins once more, against a build of oracle.c with AddressSanitizer and
UndefinedBehaviorSanitizer: an out-of-bounds read, a signed overflow or a misaligned access in the
reference itself would make every parity claim built on it worthless, and none of them needs to
change a result to be there.  Host code only; runs in a child process because the sanitizer
runtime has to be loaded before the interpreter starts."""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _gcc_file(name):
    out = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def test_oracle_pins_pass_under_address_and_ub_sanitizers():
    asan = _gcc_file("libasan.so")
    if asan is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    subprocess.check_call(["make", "-s", "-C", os.path.join(ROOT, "oracle"), "liboracle_san.so"])
    env = dict(os.environ)
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"      # the interpreter's own allocations are not the subject
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["SPECV_ORACLE_LIB"] = os.path.join(ROOT, "oracle", "liboracle_san.so")
    env["OMP_NUM_THREADS"] = "4"
    files = sorted(glob.glob(os.path.join(ROOT, "tests", "test_oracle_*.py")))
    assert files
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
