"""Builds libpwlq.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpwlq.so")
SOURCES = [os.path.join(CSRC, "pwlq_api.hip")]
HEADERS = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".h")] + [
           os.path.join(os.path.dirname(HERE), "include", "pwlq.h"),
           os.path.join(os.path.dirname(HERE), "include", "pwlq_bench.h")]

# -ffp-contract=off: the canonical code arithmetic must not be fused; fused
# operations are written explicitly where wanted.  Packed binary32 VALU forms
# are disabled for the device compile.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


# Checking configuration (CPU only): the host side of the library (argument checks,
# tensor table, workspace layout) under AddressSanitizer and
# UndefinedBehaviorSanitizer; the device code is compiled as usual.
LIB_SAN = os.path.join(HERE, "libpwlq_san.so")
HOST_SAN_FLAGS = ["-O1", "-g"] + [f for opt in ("-fsanitize=address", "-fsanitize=undefined",
                                                "-fno-sanitize-recover=all", "-fno-omit-frame-pointer")
                                  for f in ("-Xarch_host", opt)]


def hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, extra=()) -> str:
    if force or stale():
        cmd = [hipcc(), *HIPCC_FLAGS, *extra, *SOURCES, "-o", LIB]
        subprocess.run(cmd, check=True)
    return LIB


def build_sanitized() -> str:
    flags = [f for f in HIPCC_FLAGS if f != "-O3"]
    subprocess.run([hipcc(), *flags, *HOST_SAN_FLAGS, *SOURCES, "-o", LIB_SAN], check=True)
    return LIB_SAN


def sanitizer_runtime() -> str:
    """The shared AddressSanitizer runtime of the compiler hipcc drives ('' if absent)."""
    r = subprocess.run([hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"],
                       capture_output=True, text=True)
    path = r.stdout.strip()
    if os.path.isabs(path) and os.path.exists(path):
        return path
    import glob
    found = sorted(glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so"))
    return found[-1] if found else ""


if __name__ == "__main__":
    print(build(True, sys.argv[1:]))
