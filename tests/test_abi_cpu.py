"""Host-side checks that need no GPU: the library loads, exports what the
header declares, sizes workspaces sensibly and rejects bad arguments before
touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pwlq.h")
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))
                 if f.endswith(".h"))
# PWLQ_LIB: another build of the same library (the host-sanitizer configuration)
LIB = os.environ.get("PWLQ_LIB") or os.path.join(ROOT, "paper_2002_00104_amd", "libpwlq.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2002_00104_amd import build
        build.build(True)
    return ctypes.CDLL(LIB)


def declared_functions():
    text = "\n".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pwlq_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"pwlq_search", "pwlq_quantize", "pwlq_search_list", "pwlq_quantize_list"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_binding_lists_the_same_symbols():
    import importlib.util
    spec = importlib.util.find_spec("paper_2002_00104_amd.pwlq")
    src = open(spec.origin).read()
    for name in declared_functions():
        assert f'"{name}"' in src, name


def test_workspace_sizes(lib):
    f = lib.pwlq_search_workspace_bytes
    f.restype = ctypes.c_size_t
    f.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    small = f(64, 576, 4, 100, 0)
    # at least the rescaled copy of the weights and one binary32 SSE per candidate
    assert small >= 64 * 576 * 4 + 64 * 100 * 4
    assert f(38400, 4096, 4, 1000, 0) < 2 * 1024 ** 3
    assert f(64, 576, 4, 100, 1) > 0
    for bad in ((0, 5, 4, 10, 0), (5, 0, 4, 10, 0), (5, 5, 1, 10, 0), (5, 5, 9, 10, 0),
                (5, 5, 4, 0, 0), (5, 5, 4, 70000, 0), (5, 5, 4, 10, 2)):
        assert f(*bad) == 0, bad


class _Desc(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("C", ctypes.c_int64), ("K", ctypes.c_int64),
                ("group_offset", ctypes.c_int64), ("elem_offset", ctypes.c_int64)]


def test_model_level_plans_on_the_host(lib):
    """Tensor tables of 1 to 700 tensors of mixed shapes through every workspace query and,
    with a NULL workspace, through the calls themselves up to the point where they refuse."""
    import random
    rnd = random.Random(3)
    sz, ci, vp = ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p
    dp = ctypes.POINTER(_Desc)
    lib.pwlq_search_list_workspace_bytes.restype = sz
    lib.pwlq_search_list_workspace_bytes.argtypes = [dp, ci, ci, ci, ci]
    lib.pwlq_quantize_list_workspace_bytes.restype = sz
    lib.pwlq_quantize_list_workspace_bytes.argtypes = [dp, ci, ci, ci]
    lib.pwlq_select_list_workspace_bytes.restype = sz
    lib.pwlq_select_list_workspace_bytes.argtypes = [dp, ci, ci]
    lib.pwlq_mse_list_workspace_bytes.restype = sz
    lib.pwlq_mse_list_workspace_bytes.argtypes = [dp, ci, ci]
    lib.pwlq_search_list.restype = ci
    lib.pwlq_search_list.argtypes = [dp, ci, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.pwlq_search_fast_list.restype = ci
    lib.pwlq_search_fast_list.argtypes = lib.pwlq_search_list.argtypes
    fake = 0x1000   # never dereferenced
    for nt in (1, 2, 63, 64, 65, 700):
        d = (_Desc * nt)()
        g = e = 0
        for i in range(nt):
            C = rnd.choice((1, 3, 64, 1000))
            K = rnd.choice((1, 9, 64, 577, 4608, 8192, 8193, 100003))
            d[i] = _Desc(fake, C, K, g, e)
            g += C
            e += C * K
        for mode in (0, 1):
            for n in (1, 64, 1000, 2049):
                need = lib.pwlq_search_list_workspace_bytes(d, nt, 4, n, mode)
                assert need >= 4 * e
                assert lib.pwlq_search_list(d, nt, 4, n, mode, fake, fake, fake, fake, None, 0, None) == 3
                assert lib.pwlq_search_list(d, nt, 4, n, mode, fake, fake, fake, fake, fake << 8,
                                            need - 1, None) == 3
                assert lib.pwlq_search_fast_list(d, nt, 4, n, mode, fake, fake, fake, fake, fake << 8,
                                                 256, None) == 3
            assert lib.pwlq_quantize_list_workspace_bytes(d, nt, 4, mode) > 0
            assert lib.pwlq_select_list_workspace_bytes(d, nt, mode) > 0
            assert lib.pwlq_mse_list_workspace_bytes(d, nt, mode) > 0
        d[nt - 1].K = 0
        assert lib.pwlq_search_list_workspace_bytes(d, nt, 4, 100, 0) == 0


def test_bad_arguments_are_rejected_on_the_host(lib):
    lib.pwlq_last_error.restype = ctypes.c_char_p
    vp = ctypes.c_void_p
    lib.pwlq_search.restype = ctypes.c_int
    lib.pwlq_search.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                ctypes.c_int, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    fake = 0x1000  # never dereferenced: every call below fails validation first
    assert lib.pwlq_search(None, 4, 4, 4, 10, 0, fake, fake, fake, fake, fake, 1 << 20, None) == 2
    assert lib.pwlq_search(fake, 4, 4, 4, 10, 0, None, fake, fake, fake, fake, 1 << 20, None) == 2
    assert lib.pwlq_search(fake, 4, 4, 1, 10, 0, fake, fake, fake, fake, fake, 1 << 20, None) == 1
    assert lib.pwlq_search(fake, 4, 4, 4, 0, 0, fake, fake, fake, fake, fake, 1 << 20, None) == 1
    assert lib.pwlq_search(fake, 4, 4, 4, 10, 0, fake, fake, fake, fake, None, 0, None) == 3
    assert lib.pwlq_search(fake, 4, 4, 4, 10, 0, fake, fake, fake, fake, 0x1100, 16, None) == 3
    assert lib.pwlq_search(fake, 4, 4, 4, 10, 0, fake, fake, fake, fake, 0x1001, 1 << 20, None) == 3
    assert b"aligned" in lib.pwlq_last_error()
    lib.pwlq_quantize.restype = ctypes.c_int
    lib.pwlq_quantize.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                  vp, vp, vp, vp, vp, vp]
    assert lib.pwlq_quantize(fake, 4, 4, 4, 0, None, fake, fake, fake, fake, None) == 2
    assert lib.pwlq_quantize(fake, 4, 4, 9, 0, fake, fake, fake, fake, fake, None) == 1
    assert lib.pwlq_quantize(fake, 0, 4, 4, 0, fake, fake, fake, fake, fake, None) == 1


def test_wider_entry_points_reject_bad_arguments_on_the_host(lib):
    vp, i64, ci, sz, cf = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t,
                           ctypes.c_float)
    fake = 0x1000   # never dereferenced: every call below fails validation first
    lib.pwlq_search_fast.restype = ci
    lib.pwlq_search_fast.argtypes = [vp, i64, i64, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    assert lib.pwlq_search_fast(None, 4, 4, 4, 10, 0, fake, fake, fake, fake, fake, 1 << 20, None) == 2
    assert lib.pwlq_search_fast(fake, 4, 4, 4, 70000, 0, fake, fake, fake, fake, fake, 1 << 20, None) == 1

    lib.pwlq_select_workspace_bytes.restype = sz
    lib.pwlq_select_workspace_bytes.argtypes = [i64, i64, ci]
    lib.pwlq_mse_workspace_bytes.restype = sz
    lib.pwlq_mse_workspace_bytes.argtypes = [i64, i64, ci]
    # one max, one sum of squares and one sum of magnitudes per tile
    assert lib.pwlq_select_workspace_bytes(1000, 20000, 0) >= 1000 * 3 * (4 + 8 + 8)
    assert lib.pwlq_mse_workspace_bytes(1000, 20000, 0) >= 1000 * 3 * 8
    assert lib.pwlq_select_workspace_bytes(0, 5, 0) == 0
    assert lib.pwlq_mse_workspace_bytes(5, 5, 3) == 0
    lib.pwlq_select_analytic.restype = ci
    lib.pwlq_select_analytic.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, sz, vp]
    assert lib.pwlq_select_analytic(fake, 4, 4, 0, 3, fake, fake, fake, 1 << 20, None) == 1
    assert lib.pwlq_select_analytic(fake, 4, 4, 0, -1, fake, fake, fake, 1 << 20, None) == 1
    assert lib.pwlq_select_analytic(fake, 4, 4, 0, 1, None, fake, fake, 1 << 20, None) == 2
    assert lib.pwlq_select_analytic(fake, 4, 4, 0, 1, fake, fake, None, 0, None) == 3
    lib.pwlq_mse.restype = ci
    lib.pwlq_mse.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp, sz, vp]
    assert lib.pwlq_mse(fake, 4, 4, 1, 0, fake, fake, fake, fake, 1 << 20, None) == 1
    assert lib.pwlq_mse(fake, 4, 4, 4, 0, fake, None, fake, fake, 1 << 20, None) == 2
    assert lib.pwlq_mse(fake, 4, 4, 4, 0, fake, fake, fake, fake, 8, None) == 3

    lib.pwlq_linear_workspace_bytes.restype = sz
    lib.pwlq_linear_workspace_bytes.argtypes = [i64]
    assert lib.pwlq_linear_workspace_bytes(1000) >= 4000
    assert lib.pwlq_linear_workspace_bytes(0) == 0
    lib.pwlq_linear_i8.restype = ci
    lib.pwlq_linear_i8.argtypes = [vp, i64, i64, cf, cf, vp, vp, i64, ci, vp, vp, vp, vp, vp, sz, vp]
    ok = (fake, 8, 128, 1.0, 0.0, fake, fake, 8, 4, fake, fake, fake, None, fake, 1 << 20, None)

    def call(**kw):
        names = ("xq", "M", "K", "s_x", "z_x", "codes", "flags", "N", "bits", "p", "m", "y", "acc",
                 "ws", "ws_bytes", "stream")
        a = dict(zip(names, ok))
        a.update(kw)
        return lib.pwlq_linear_i8(*[a[n] for n in names])

    assert call(K=100) == 1                       # K must be a multiple of 16
    assert call(bits=1) == 1
    assert call(M=0) == 1
    assert call(xq=None) == 2
    assert call(y=None) == 2
    assert call(codes=0x1008) == 1                # packed codes must be 16-byte aligned
    assert call(flags=0x1001) == 1
    assert call(ws=None) == 3
    assert call(ws_bytes=4) == 3
    assert call(ws=0x1010) == 3

    lib.pwlq_profile_ms.restype = ctypes.c_double
    lib.pwlq_profile_ms.argtypes = [ci, ci]
    assert lib.pwlq_profile_ms(0, 0) == -1.0       # nothing recorded without a GPU
    assert lib.pwlq_profile_ms(9, 0) == -1.0


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more exits with a message and no JSON line."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert "{" not in r.stdout


def test_header_is_plain_c(tmp_path):
    """Every header under include/ compiles as C99 on its own (no HIP or C++ needed by a caller)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc not found")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = "\n".join(re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S) for h in HEADERS)
    names = sorted(set(re.findall(r"\b(pwlq_[a-z0-9_]+)\s*\(", text)))
    assert len(names) > 20
    src = tmp_path / "use_header.c"
    body = "\n".join(f"    table[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text("".join(f'#include "{os.path.basename(h)}"\n' for h in HEADERS) +
                   f"void (*table[{len(names)}])(void);\n"
                   "void fill(void)\n{\n" + body + "\n}\n")
    r = subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-c",
                        "-I", os.path.join(root, "include"), str(src), "-o", str(tmp_path / "use_header.o")],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stderr
