"""The host side of libpwlq under AddressSanitizer and UndefinedBehaviorSanitizer
(CPU only; the device code is compiled as usual and never runs here).

The library is built a second time with the sanitizers applied to the host
pass only, and the host-side tests (argument checks, tensor tables, workspace
layout, exported symbols) run again against that build in a child interpreter
that preloads the sanitizer runtime."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_side_passes_under_asan_and_ubsan():
    from paper_2002_00104_amd import build
    runtime = build.sanitizer_runtime()
    if not runtime:
        pytest.skip("the compiler has no shared AddressSanitizer runtime")
    lib = build.build_sanitized()
    env = dict(os.environ)
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["PWLQ_LIB"] = lib
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        "tests/test_abi_cpu.py", "-k", "not more_than_one_gpu and not plain_c"],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    assert "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, tail
