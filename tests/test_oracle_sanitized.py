"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

`oracle/pwlq_oracle.c` is compiled a second time with
`-fsanitize=address,undefined -fno-sanitize-recover=all -O1` and every oracle
pin (the Eq.3 table, the brute-force comparisons, pack round trips, argument
checks, the selectors, the integer inner product) is run again through that
library in a child interpreter that preloads the sanitizer runtime: any
out-of-bounds access, signed overflow, misaligned or invalid shift in the
oracle ends the child with a report.  A second child calls the library with an
output buffer that is too short, to show that the configuration does catch
such an access.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_pins.py", "tests/test_oracle_selectors.py",
             "tests/test_oracle_linear.py"]


def _runtime():
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc not found")
    path = subprocess.run([gcc, "-print-file-name=libasan.so"], capture_output=True,
                          text=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip("gcc has no shared AddressSanitizer runtime")
    return path


def _env(runtime):
    env = dict(os.environ)
    # the sanitizer runtime must come first among the preloaded libraries; whatever the
    # environment already preloads stays behind it
    env["LD_PRELOAD"] = runtime + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["PWLQ_REF_SANITIZE"] = "1"
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    env["PYTHONPATH"] = ROOT + (os.pathsep + env["PYTHONPATH"] if env.get("PYTHONPATH") else "")
    return env


@pytest.fixture(scope="module")
def sanitized():
    runtime = _runtime()
    from oracle import pwlq_ref
    path = pwlq_ref.build(force=True, sanitize=True)
    return runtime, path


def test_oracle_pins_pass_under_asan_and_ubsan(sanitized):
    runtime, path = sanitized
    env = _env(runtime)
    which = subprocess.run([sys.executable, "-c",
                            "from oracle import pwlq_ref as R; R.lib(); print(R.loaded_path())"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert which.returncode == 0, which.stderr[-2000:]
    assert which.stdout.strip() == path               # the child really runs the checked build
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        *PIN_FILES], cwd=ROOT, env=env, capture_output=True, text=True,
                       timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "failed" not in r.stdout, tail
    assert "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, tail


def test_the_configuration_catches_an_out_of_bounds_write(sanitized):
    """pwlq_ref_pack writes ceil(n*bits/8) bytes; give it one byte less."""
    runtime, _ = sanitized
    code = (
        "import ctypes, numpy as np\n"
        "from oracle import pwlq_ref as R\n"
        "L = R.lib()\n"
        "n, bits = 64, 4\n"
        "codes = np.zeros(n, np.uint8); flags = np.zeros(n, np.uint8)\n"
        "pc = np.empty(n * bits // 8 - 1, np.uint8); pf = np.empty(n // 8, np.uint8)\n"
        "u8 = ctypes.POINTER(ctypes.c_uint8)\n"
        "L.pwlq_ref_pack(codes.ctypes.data_as(u8), flags.ctypes.data_as(u8), n, bits,\n"
        "                pc.ctypes.data_as(u8), pf.ctypes.data_as(u8))\n"
        "print('returned')\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=_env(runtime),
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "AddressSanitizer" in r.stderr and "heap-buffer-overflow" in r.stderr, r.stderr[-2000:]
    assert "returned" not in r.stdout
