"""ctypes loader for the CPU oracle (``pwlq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by
the benchmark's cpu_baseline leg.  The product package never imports this
module, and this module never imports the product's HIP binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pwlq_oracle.c")
_LIB = os.path.join(_HERE, "libpwlq_ref.so")

PER_CHANNEL = 0
PER_TENSOR = 1

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-shared", "-fPIC", "-Wall", "-Wextra"]

# Checking configuration: the same source under AddressSanitizer and
# UndefinedBehaviorSanitizer, in a library of its own.  A process that sets
# PWLQ_REF_SANITIZE=1 (and preloads gcc's libasan.so) loads that one instead.
_LIB_SAN = os.path.join(_HERE, "libpwlq_ref_san.so")
SAN_CFLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
              "-fno-sanitize-recover=all"] + [f for f in CFLAGS if f != "-O2"]
SANITIZE = os.environ.get("PWLQ_REF_SANITIZE") == "1"


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared object."""
    out, flags = (_LIB_SAN, SAN_CFLAGS) if sanitize else (_LIB, CFLAGS)
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        cmd = ["gcc", *flags, _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)
    return out


_lib: Optional[ctypes.CDLL] = None
_loaded: Optional[str] = None


def loaded_path() -> Optional[str]:
    """Path of the shared object this process has loaded (None before the first call)."""
    return _loaded


def lib() -> ctypes.CDLL:
    global _lib, _loaded
    if _lib is None:
        _loaded = build(sanitize=SANITIZE)
        L = ctypes.CDLL(_loaded)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        bp = ctypes.POINTER(ctypes.c_uint8)
        L.pwlq_ref_search.restype = ctypes.c_int
        L.pwlq_ref_search.argtypes = [fp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_int, fp, fp, ip, dp, dp]
        L.pwlq_ref_quantize.restype = ctypes.c_int
        L.pwlq_ref_quantize.argtypes = [fp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                        ctypes.c_int, fp, fp, bp, bp, fp]
        L.pwlq_ref_num_threads.restype = ctypes.c_int
        L.pwlq_ref_pack.restype = ctypes.c_int
        L.pwlq_ref_pack.argtypes = [bp, bp, ctypes.c_int64, ctypes.c_int, bp, bp]
        L.pwlq_ref_unpack.restype = ctypes.c_int
        L.pwlq_ref_unpack.argtypes = [bp, bp, ctypes.c_int64, ctypes.c_int, bp, bp]
        L.pwlq_ref_select_analytic.restype = ctypes.c_int
        L.pwlq_ref_select_analytic.argtypes = [fp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int,
                                               ctypes.c_int, fp, fp]
        L.pwlq_ref_mse.restype = ctypes.c_int
        L.pwlq_ref_mse.argtypes = [fp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                   fp, fp, dp]
        L.pwlq_ref_linear.restype = ctypes.c_int
        L.pwlq_ref_linear.argtypes = [ctypes.POINTER(ctypes.c_int8), ctypes.c_int64, ctypes.c_int64,
                                      ctypes.c_float, ctypes.c_float, bp, bp, ctypes.c_int64,
                                      ctypes.c_int, fp, fp, ctypes.POINTER(ctypes.c_int64), dp]
        _lib = L
    return _lib


def linear(xq: np.ndarray, s_x: float, z_x: float, codes: np.ndarray, flags: np.ndarray, bits: int,
           p: np.ndarray, m: np.ndarray, want_acc: bool = False):
    """Section 4's integer inner products.  xq int8 [M, K]; codes, flags uint8 [N, K]
    (one byte each); p, m float32 [N].  Returns y float64 [M, N] (and the three
    integer sums int64 [3, M, N])."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    flags = np.ascontiguousarray(flags, dtype=np.uint8)
    p = np.ascontiguousarray(p, dtype=np.float32)
    m = np.ascontiguousarray(m, dtype=np.float32)
    M, K = xq.shape
    N = codes.shape[0]
    if codes.shape != (N, K) or flags.shape != (N, K) or p.shape != (N,) or m.shape != (N,):
        raise ValueError("shape mismatch")
    y = np.empty((M, N), np.float64)
    acc = np.empty((3, M, N), np.int64) if want_acc else None
    rc = lib().pwlq_ref_linear(_ptr(xq, ctypes.c_int8), M, K, s_x, z_x,
                               _ptr(codes, ctypes.c_uint8), _ptr(flags, ctypes.c_uint8), N, bits,
                               _ptr(p, ctypes.c_float), _ptr(m, ctypes.c_float),
                               _ptr(acc, ctypes.c_int64) if want_acc else None,
                               _ptr(y, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"pwlq_ref_linear status {rc}")
    return (y, acc) if want_acc else y


GAUSS_FIT, GAUSS_SOLVE, LAPLACE_SOLVE = 0, 1, 2


def select_analytic(w: np.ndarray, selector: int, mode: int = PER_CHANNEL):
    """The paper's analytic breakpoint selectors.  Returns (p f32 [G], m f32 [G])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    C, K = w.shape
    G = C if mode == PER_CHANNEL else 1
    p = np.empty(G, np.float32)
    m = np.empty(G, np.float32)
    rc = lib().pwlq_ref_select_analytic(_ptr(w, ctypes.c_float), C, K, mode, selector,
                                        _ptr(p, ctypes.c_float), _ptr(m, ctypes.c_float))
    if rc != 0:
        raise ValueError(f"pwlq_ref_select_analytic status {rc}")
    return p, m


def mse(w: np.ndarray, bits: int, p: np.ndarray, m: np.ndarray, mode: int = PER_CHANNEL):
    """Mean squared quantization error for given (m, p) per group (float64 [G])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    C, K = w.shape
    G = C if mode == PER_CHANNEL else 1
    p = np.ascontiguousarray(p, dtype=np.float32)
    m = np.ascontiguousarray(m, dtype=np.float32)
    out = np.empty(G, np.float64)
    rc = lib().pwlq_ref_mse(_ptr(w, ctypes.c_float), C, K, bits, mode, _ptr(p, ctypes.c_float),
                            _ptr(m, ctypes.c_float), _ptr(out, ctypes.c_double))
    if rc != 0:
        raise ValueError(f"pwlq_ref_mse status {rc}")
    return out


def _ptr(a: np.ndarray, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def num_threads() -> int:
    return int(lib().pwlq_ref_num_threads())


def search(w: np.ndarray, bits: int, n_cand: int, mode: int = PER_CHANNEL,
           want_curve: bool = False):
    """w: [C, K] float32.  Returns dict(p_star, m, k_star, mse[, curve])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim != 2:
        raise ValueError("w must be [C, K]")
    C, K = w.shape
    G = C if mode == PER_CHANNEL else 1
    p_star = np.empty(G, np.float32)
    m = np.empty(G, np.float32)
    k_star = np.empty(G, np.int32)
    mse = np.empty(G, np.float64)
    curve = np.empty((G, n_cand), np.float64) if want_curve else None
    rc = lib().pwlq_ref_search(
        _ptr(w, ctypes.c_float), C, K, bits, n_cand, mode,
        _ptr(p_star, ctypes.c_float), _ptr(m, ctypes.c_float),
        _ptr(k_star, ctypes.c_int32), _ptr(mse, ctypes.c_double),
        _ptr(curve, ctypes.c_double) if want_curve else None)
    if rc != 0:
        raise ValueError(f"pwlq_ref_search status {rc}")
    out = dict(p_star=p_star, m=m, k_star=k_star, mse=mse)
    if want_curve:
        out["curve"] = curve
    return out


def quantize(w: np.ndarray, bits: int, p_star: np.ndarray, m: np.ndarray,
             mode: int = PER_CHANNEL) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Returns (codes u8, flags u8, w_hat f32), each shaped like w."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    C, K = w.shape
    G = C if mode == PER_CHANNEL else 1
    p_star = np.ascontiguousarray(p_star, dtype=np.float32)
    m = np.ascontiguousarray(m, dtype=np.float32)
    if p_star.shape != (G,) or m.shape != (G,):
        raise ValueError("p_star and m must have one entry per group")
    codes = np.empty((C, K), np.uint8)
    flags = np.empty((C, K), np.uint8)
    w_hat = np.empty((C, K), np.float32)
    rc = lib().pwlq_ref_quantize(
        _ptr(w, ctypes.c_float), C, K, bits, mode,
        _ptr(p_star, ctypes.c_float), _ptr(m, ctypes.c_float),
        _ptr(codes, ctypes.c_uint8), _ptr(flags, ctypes.c_uint8),
        _ptr(w_hat, ctypes.c_float))
    if rc != 0:
        raise ValueError(f"pwlq_ref_quantize status {rc}")
    return codes, flags, w_hat


def pack(codes: np.ndarray, flags: np.ndarray, bits: int) -> Tuple[np.ndarray, np.ndarray]:
    """Bit-packs a tensor's codes and flags (any shape, row-major order)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8).reshape(-1)
    flags = np.ascontiguousarray(flags, dtype=np.uint8).reshape(-1)
    n = codes.size
    pc = np.empty((n * bits + 7) // 8, np.uint8)
    pf = np.empty((n + 7) // 8, np.uint8)
    rc = lib().pwlq_ref_pack(_ptr(codes, ctypes.c_uint8), _ptr(flags, ctypes.c_uint8), n, bits,
                             _ptr(pc, ctypes.c_uint8), _ptr(pf, ctypes.c_uint8))
    if rc != 0:
        raise ValueError(f"pwlq_ref_pack status {rc}")
    return pc, pf


def unpack(packed_codes: np.ndarray, packed_flags: np.ndarray, count: int,
           bits: int) -> Tuple[np.ndarray, np.ndarray]:
    pc = np.ascontiguousarray(packed_codes, dtype=np.uint8)
    pf = np.ascontiguousarray(packed_flags, dtype=np.uint8)
    codes = np.empty(count, np.uint8)
    flags = np.empty(count, np.uint8)
    rc = lib().pwlq_ref_unpack(_ptr(pc, ctypes.c_uint8), _ptr(pf, ctypes.c_uint8), count, bits,
                               _ptr(codes, ctypes.c_uint8), _ptr(flags, ctypes.c_uint8))
    if rc != 0:
        raise ValueError(f"pwlq_ref_unpack status {rc}")
    return codes, flags
