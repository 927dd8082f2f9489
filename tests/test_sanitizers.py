"""The oracle and the host side of the C ABI under AddressSanitizer + UndefinedBehaviorSanitizer.

Both are rebuilt with clang's host sanitizers (device code is untouched) into libraries of their
own, and the oracle pins and the ABI tests run against those in a child Python process that
preloads the sanitizer runtime.  No GPU is used: the ABI tests only exercise argument validation
and the scratch layout arithmetic.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_and_abi_checks_under_host_sanitizers():
    sys.path.insert(0, ROOT)
    from paper_2605_08840_amd import build as hip_build
    rt = hip_build.asan_runtime()
    if not rt:
        pytest.skip("the toolchain ships no shared AddressSanitizer runtime")
    lib = hip_build.build(verbose=False, sanitize=True)
    env = dict(os.environ)
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["RESTKV_ORACLE_SANITIZE"] = "1"
    env["RESTKV_LIB"] = lib
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_abi.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=900)
    out = r.stdout.decode(errors="replace")
    assert r.returncode == 0, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert " passed" in out
