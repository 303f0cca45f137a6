"""ctypes binding over libpwlq.so: argument marshalling only.

Every step of the search and of the quantizer runs in the library's HIP
kernels; PyTorch is used for device memory and for the current stream.  There
is no fallback: if the shared library is missing the import of this module
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import torch

PER_CHANNEL = 0
PER_TENSOR = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpwlq.so")

EXPORTS = (
    "pwlq_search_workspace_bytes", "pwlq_search", "pwlq_quantize",
    "pwlq_search_list_workspace_bytes", "pwlq_search_list",
    "pwlq_search_fast", "pwlq_search_fast_list", "pwlq_search_static",
    "pwlq_quantize_list_workspace_bytes", "pwlq_quantize_list",
    "pwlq_packed_code_bytes", "pwlq_packed_flag_bytes", "pwlq_quantize_packed",
    "pwlq_quantize_packed_list",
    "pwlq_select_workspace_bytes", "pwlq_select_list_workspace_bytes", "pwlq_select_analytic",
    "pwlq_select_analytic_list",
    "pwlq_mse_workspace_bytes", "pwlq_mse_list_workspace_bytes", "pwlq_mse", "pwlq_mse_list",
    "pwlq_linear_workspace_bytes", "pwlq_linear_i8",
    "pwlq_last_error", "pwlq_last_search_shape", "pwlq_profile_enable",
    "pwlq_profile_last_ms", "pwlq_profile_ms", "pwlq_kernel_name", "pwlq_last_search_kernel",
    "pwlq_set_small_call_tiles",
)


class TensorDesc(ctypes.Structure):
    _fields_ = [("w", ctypes.c_void_p), ("C", ctypes.c_int64), ("K", ctypes.c_int64),
                ("group_offset", ctypes.c_int64), ("elem_offset", ctypes.c_int64)]


class PwlqError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libpwlq status {status}: {text}")
        self.status = status


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2002_00104_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    dp = ctypes.POINTER(TensorDesc)
    lib.pwlq_search_workspace_bytes.restype = sz
    lib.pwlq_search_workspace_bytes.argtypes = [i64, i64, ci, ci, ci]
    lib.pwlq_search.restype = ci
    lib.pwlq_search.argtypes = [vp, i64, i64, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.pwlq_search_fast.restype = ci
    lib.pwlq_search_fast.argtypes = lib.pwlq_search.argtypes
    lib.pwlq_search_static.restype = ci
    lib.pwlq_search_static.argtypes = [vp, i64, i64, ci, ci, ci, vp, vp, vp, vp, vp]
    lib.pwlq_quantize.restype = ci
    lib.pwlq_quantize.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.pwlq_search_list_workspace_bytes.restype = sz
    lib.pwlq_search_list_workspace_bytes.argtypes = [dp, ci, ci, ci, ci]
    lib.pwlq_search_list.restype = ci
    lib.pwlq_search_list.argtypes = [dp, ci, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.pwlq_search_fast_list.restype = ci
    lib.pwlq_search_fast_list.argtypes = lib.pwlq_search_list.argtypes
    lib.pwlq_quantize_list_workspace_bytes.restype = sz
    lib.pwlq_quantize_list_workspace_bytes.argtypes = [dp, ci, ci, ci]
    lib.pwlq_quantize_list.restype = ci
    lib.pwlq_quantize_list.argtypes = [dp, ci, ci, ci, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.pwlq_packed_code_bytes.restype = sz
    lib.pwlq_packed_code_bytes.argtypes = [i64, ci]
    lib.pwlq_packed_flag_bytes.restype = sz
    lib.pwlq_packed_flag_bytes.argtypes = [i64]
    lib.pwlq_quantize_packed.restype = ci
    lib.pwlq_quantize_packed.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp, vp, vp]
    lib.pwlq_quantize_packed_list.restype = ci
    lib.pwlq_quantize_packed_list.argtypes = [dp, ci, ci, ci, vp, vp, vp, ctypes.POINTER(i64), vp,
                                              ctypes.POINTER(i64), vp, vp, sz, vp]
    lib.pwlq_select_workspace_bytes.restype = sz
    lib.pwlq_select_workspace_bytes.argtypes = [i64, i64, ci]
    lib.pwlq_select_list_workspace_bytes.restype = sz
    lib.pwlq_select_list_workspace_bytes.argtypes = [dp, ci, ci]
    lib.pwlq_select_analytic.restype = ci
    lib.pwlq_select_analytic.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, sz, vp]
    lib.pwlq_select_analytic_list.restype = ci
    lib.pwlq_select_analytic_list.argtypes = [dp, ci, ci, ci, vp, vp, vp, sz, vp]
    lib.pwlq_mse_workspace_bytes.restype = sz
    lib.pwlq_mse_workspace_bytes.argtypes = [i64, i64, ci]
    lib.pwlq_mse_list_workspace_bytes.restype = sz
    lib.pwlq_mse_list_workspace_bytes.argtypes = [dp, ci, ci]
    lib.pwlq_mse.restype = ci
    lib.pwlq_mse.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, vp, sz, vp]
    lib.pwlq_mse_list.restype = ci
    lib.pwlq_mse_list.argtypes = [dp, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    lib.pwlq_linear_workspace_bytes.restype = sz
    lib.pwlq_linear_workspace_bytes.argtypes = [i64]
    lib.pwlq_linear_i8.restype = ci
    lib.pwlq_linear_i8.argtypes = [vp, i64, i64, ctypes.c_float, ctypes.c_float, vp, vp, i64, ci,
                                   vp, vp, vp, vp, vp, sz, vp]
    lib.pwlq_last_error.restype = ctypes.c_char_p
    lib.pwlq_last_error.argtypes = []
    lib.pwlq_last_search_shape.restype = None
    lib.pwlq_last_search_shape.argtypes = [ctypes.POINTER(i64)] * 3
    lib.pwlq_profile_enable.restype = None
    lib.pwlq_profile_enable.argtypes = [ci]
    lib.pwlq_profile_last_ms.restype = ctypes.c_double
    lib.pwlq_profile_last_ms.argtypes = [ci]
    lib.pwlq_profile_ms.restype = ctypes.c_double
    lib.pwlq_profile_ms.argtypes = [ci, ci]
    lib.pwlq_kernel_name.restype = ctypes.c_char_p
    lib.pwlq_kernel_name.argtypes = [ci]
    lib.pwlq_last_search_kernel.restype = ctypes.c_char_p
    lib.pwlq_last_search_kernel.argtypes = []
    lib.pwlq_set_small_call_tiles.restype = ctypes.c_int
    lib.pwlq_set_small_call_tiles.argtypes = [ctypes.c_int]
    return lib


lib = _load()


def _check(status: int) -> None:
    if status != 0:
        raise PwlqError(status, lib.pwlq_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev32(w: torch.Tensor) -> torch.Tensor:
    if not (w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and w.dim() == 2):
        raise ValueError("weights must be a contiguous float32 [C, K] tensor on the GPU")
    return w


def _n_groups(C: int, mode: int) -> int:
    return C if mode == PER_CHANNEL else 1


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def search_workspace_bytes(C: int, K: int, bits: int, n_cand: int, mode: int) -> int:
    return int(lib.pwlq_search_workspace_bytes(C, K, bits, n_cand, mode))


def search(w: torch.Tensor, bits: int, n_cand: int, mode: int = PER_CHANNEL,
           workspace: Optional[torch.Tensor] = None, fast: bool = False) -> Dict[str, torch.Tensor]:
    """pwlq_search (or pwlq_search_fast) on one [C, K] tensor.
    Returns p_star, m, k_star, mse (device)."""
    w = _dev32(w)
    C, K = w.shape
    G = _n_groups(C, mode)
    if workspace is None:
        workspace = _workspace(search_workspace_bytes(C, K, bits, n_cand, mode), w.device)
    out = dict(p_star=torch.empty(G, dtype=torch.float32, device=w.device),
               m=torch.empty(G, dtype=torch.float32, device=w.device),
               k_star=torch.empty(G, dtype=torch.int32, device=w.device),
               mse=torch.empty(G, dtype=torch.float64, device=w.device))
    fn = lib.pwlq_search_fast if fast else lib.pwlq_search
    _check(fn(w.data_ptr(), C, K, bits, n_cand, mode, out["p_star"].data_ptr(),
              out["m"].data_ptr(), out["k_star"].data_ptr(), out["mse"].data_ptr(),
              workspace.data_ptr(), workspace.numel(), _stream()))
    return out


STATIC_SCRATCH_BYTES = 32 << 20


def search_static(w: torch.Tensor, bits: int, n_cand: int, mode: int = PER_CHANNEL,
                  out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """pwlq_search_static on one [C, K] tensor: the search with the library's own
    scratch buffer.  With `out` given (see alloc_search_outputs) this binding
    allocates nothing either."""
    w = _dev32(w)
    C, K = w.shape
    if out is None:
        out = alloc_search_outputs(_n_groups(C, mode), w.device)
    _check(lib.pwlq_search_static(w.data_ptr(), C, K, bits, n_cand, mode, out["p_star"].data_ptr(),
                                  out["m"].data_ptr(), out["k_star"].data_ptr(),
                                  out["mse"].data_ptr(), _stream()))
    return out


def quantize(w: torch.Tensor, bits: int, p_star: torch.Tensor, m: torch.Tensor,
             mode: int = PER_CHANNEL):
    """pwlq_quantize on one [C, K] tensor.  Returns (codes u8, flags u8, w_hat f32)."""
    w = _dev32(w)
    C, K = w.shape
    G = _n_groups(C, mode)
    for t in (p_star, m):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == G):
            raise ValueError("p_star and m must be float32 device tensors with one entry per group")
    codes = torch.empty((C, K), dtype=torch.uint8, device=w.device)
    flags = torch.empty((C, K), dtype=torch.uint8, device=w.device)
    w_hat = torch.empty((C, K), dtype=torch.float32, device=w.device)
    _check(lib.pwlq_quantize(w.data_ptr(), C, K, bits, mode, p_star.data_ptr(), m.data_ptr(),
                             codes.data_ptr(), flags.data_ptr(), w_hat.data_ptr(), _stream()))
    return codes, flags, w_hat


class TensorList:
    """Descriptor table for the model-level calls: tensors laid out back to back
    in the per-group and per-element arrays, in the order given."""

    def __init__(self, tensors: Sequence[torch.Tensor], mode: int):
        self.tensors: List[torch.Tensor] = [_dev32(t) for t in tensors]
        self.mode = mode
        self.device = self.tensors[0].device
        self.desc = (TensorDesc * len(self.tensors))()
        g = e = 0
        self.group_offsets: List[int] = []
        self.elem_offsets: List[int] = []
        for i, t in enumerate(self.tensors):
            C, K = t.shape
            self.desc[i] = TensorDesc(t.data_ptr(), C, K, g, e)
            self.group_offsets.append(g)
            self.elem_offsets.append(e)
            g += _n_groups(C, mode)
            e += C * K
        self.n_groups = g
        self.n_elements = e

    def __len__(self) -> int:
        return len(self.tensors)

    def group_counts(self, select: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Elements per group (float64, device), in per-group array order."""
        if not hasattr(self, "_counts"):
            parts = []
            for t in self.tensors:
                C, K = t.shape
                G = _n_groups(C, self.mode)
                parts.append(torch.full((G,), float(C * K // G), dtype=torch.float64))
            self._counts = torch.cat(parts).to(self.device)
        return self._counts if select is None else self._counts[select]


def search_list_workspace_bytes(tl: TensorList, bits: int, n_cand: int) -> int:
    return int(lib.pwlq_search_list_workspace_bytes(tl.desc, len(tl), bits, n_cand, tl.mode))


def search_list(tl: TensorList, bits: int, n_cand: int,
                workspace: Optional[torch.Tensor] = None,
                out: Optional[Dict[str, torch.Tensor]] = None,
                fast: bool = False) -> Dict[str, torch.Tensor]:
    if workspace is None:
        workspace = _workspace(search_list_workspace_bytes(tl, bits, n_cand), tl.device)
    if out is None:
        out = alloc_search_outputs(tl.n_groups, tl.device)
    fn = lib.pwlq_search_fast_list if fast else lib.pwlq_search_list
    _check(fn(tl.desc, len(tl), bits, n_cand, tl.mode, out["p_star"].data_ptr(),
              out["m"].data_ptr(), out["k_star"].data_ptr(), out["mse"].data_ptr(),
              workspace.data_ptr(), workspace.numel(), _stream()))
    return out


def alloc_search_outputs(G: int, device) -> Dict[str, torch.Tensor]:
    return dict(p_star=torch.empty(G, dtype=torch.float32, device=device),
                m=torch.empty(G, dtype=torch.float32, device=device),
                k_star=torch.empty(G, dtype=torch.int32, device=device),
                mse=torch.empty(G, dtype=torch.float64, device=device))


def quantize_list_workspace_bytes(tl: TensorList, bits: int) -> int:
    return int(lib.pwlq_quantize_list_workspace_bytes(tl.desc, len(tl), bits, tl.mode))


def alloc_quantize_outputs(n_elements: int, device):
    return (torch.empty(n_elements, dtype=torch.uint8, device=device),
            torch.empty(n_elements, dtype=torch.uint8, device=device),
            torch.empty(n_elements, dtype=torch.float32, device=device))


def quantize_list(tl: TensorList, bits: int, p_star: torch.Tensor, m: torch.Tensor,
                  workspace: Optional[torch.Tensor] = None, out=None):
    if workspace is None:
        workspace = _workspace(quantize_list_workspace_bytes(tl, bits), tl.device)
    if out is None:
        out = alloc_quantize_outputs(tl.n_elements, tl.device)
    codes, flags, w_hat = out
    _check(lib.pwlq_quantize_list(tl.desc, len(tl), bits, tl.mode, p_star.data_ptr(), m.data_ptr(),
                                  codes.data_ptr(), flags.data_ptr(), w_hat.data_ptr(),
                                  workspace.data_ptr(), workspace.numel(), _stream()))
    return codes, flags, w_hat


def packed_code_bytes(count: int, bits: int) -> int:
    return int(lib.pwlq_packed_code_bytes(count, bits))


def packed_flag_bytes(count: int) -> int:
    return int(lib.pwlq_packed_flag_bytes(count))


def quantize_packed(w: torch.Tensor, bits: int, p_star: torch.Tensor, m: torch.Tensor,
                    mode: int = PER_CHANNEL, want_w_hat: bool = True):
    """pwlq_quantize_packed on one [C, K] tensor.
    Returns (packed_codes u8, packed_flags u8, w_hat f32 or None)."""
    w = _dev32(w)
    C, K = w.shape
    n = C * K
    pc = torch.empty(packed_code_bytes(n, bits), dtype=torch.uint8, device=w.device)
    pf = torch.empty(packed_flag_bytes(n), dtype=torch.uint8, device=w.device)
    w_hat = torch.empty((C, K), dtype=torch.float32, device=w.device) if want_w_hat else None
    _check(lib.pwlq_quantize_packed(w.data_ptr(), C, K, bits, mode, p_star.data_ptr(),
                                    m.data_ptr(), pc.data_ptr(), pf.data_ptr(),
                                    w_hat.data_ptr() if want_w_hat else None, _stream()))
    return pc, pf, w_hat


class PackedLayout:
    """Byte offsets of every tensor's code and flag stream inside two shared
    buffers; each stream starts on a 4-byte boundary."""

    def __init__(self, tl: "TensorList", bits: int):
        n = len(tl)
        self.code_off = (ctypes.c_int64 * n)()
        self.flag_off = (ctypes.c_int64 * n)()
        c = f = 0
        for i, t in enumerate(tl.tensors):
            self.code_off[i] = c
            self.flag_off[i] = f
            c += (packed_code_bytes(t.numel(), bits) + 3) // 4 * 4
            f += (packed_flag_bytes(t.numel()) + 3) // 4 * 4
        self.code_bytes = c
        self.flag_bytes = f


def quantize_packed_list(tl: "TensorList", bits: int, p_star: torch.Tensor, m: torch.Tensor,
                         layout: Optional[PackedLayout] = None, want_w_hat: bool = False,
                         workspace: Optional[torch.Tensor] = None, out=None):
    if layout is None:
        layout = PackedLayout(tl, bits)
    if workspace is None:
        workspace = _workspace(quantize_list_workspace_bytes(tl, bits), tl.device)
    if out is None:
        out = (torch.empty(max(layout.code_bytes, 4), dtype=torch.uint8, device=tl.device),
               torch.empty(max(layout.flag_bytes, 4), dtype=torch.uint8, device=tl.device),
               torch.empty(tl.n_elements, dtype=torch.float32, device=tl.device)
               if want_w_hat else None)
    pc, pf, w_hat = out
    _check(lib.pwlq_quantize_packed_list(tl.desc, len(tl), bits, tl.mode, p_star.data_ptr(),
                                         m.data_ptr(), pc.data_ptr(), layout.code_off,
                                         pf.data_ptr(), layout.flag_off,
                                         w_hat.data_ptr() if w_hat is not None else None,
                                         workspace.data_ptr(), workspace.numel(), _stream()))
    return pc, pf, w_hat, layout


GAUSS_FIT, GAUSS_SOLVE, LAPLACE_SOLVE = 0, 1, 2


def select_analytic(w: torch.Tensor, selector: int, mode: int = PER_CHANNEL,
                    workspace: Optional[torch.Tensor] = None):
    """pwlq_select_analytic on one [C, K] tensor.  Returns (p f32 [G], m f32 [G])."""
    w = _dev32(w)
    C, K = w.shape
    G = _n_groups(C, mode)
    if workspace is None:
        workspace = _workspace(lib.pwlq_select_workspace_bytes(C, K, mode), w.device)
    p = torch.empty(G, dtype=torch.float32, device=w.device)
    m = torch.empty(G, dtype=torch.float32, device=w.device)
    _check(lib.pwlq_select_analytic(w.data_ptr(), C, K, mode, selector, p.data_ptr(),
                                    m.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                    _stream()))
    return p, m


def select_list_workspace_bytes(tl: "TensorList") -> int:
    return int(lib.pwlq_select_list_workspace_bytes(tl.desc, len(tl), tl.mode))


def select_analytic_list(tl: "TensorList", selector: int,
                         workspace: Optional[torch.Tensor] = None, out=None):
    if workspace is None:
        workspace = _workspace(select_list_workspace_bytes(tl), tl.device)
    if out is None:
        out = (torch.empty(tl.n_groups, dtype=torch.float32, device=tl.device),
               torch.empty(tl.n_groups, dtype=torch.float32, device=tl.device))
    p, m = out
    _check(lib.pwlq_select_analytic_list(tl.desc, len(tl), tl.mode, selector, p.data_ptr(),
                                         m.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                         _stream()))
    return p, m


def mse(w: torch.Tensor, bits: int, p: torch.Tensor, m: torch.Tensor, mode: int = PER_CHANNEL,
        workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """pwlq_mse on one [C, K] tensor.  Returns f64 [G]."""
    w = _dev32(w)
    C, K = w.shape
    G = _n_groups(C, mode)
    for t in (p, m):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == G):
            raise ValueError("p and m must be float32 device tensors with one entry per group")
    if workspace is None:
        workspace = _workspace(lib.pwlq_mse_workspace_bytes(C, K, mode), w.device)
    out = torch.empty(G, dtype=torch.float64, device=w.device)
    _check(lib.pwlq_mse(w.data_ptr(), C, K, bits, mode, p.data_ptr(), m.data_ptr(),
                        out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()))
    return out


def mse_list_workspace_bytes(tl: "TensorList") -> int:
    return int(lib.pwlq_mse_list_workspace_bytes(tl.desc, len(tl), tl.mode))


def mse_list(tl: "TensorList", bits: int, p: torch.Tensor, m: torch.Tensor,
             workspace: Optional[torch.Tensor] = None,
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if workspace is None:
        workspace = _workspace(mse_list_workspace_bytes(tl), tl.device)
    if out is None:
        out = torch.empty(tl.n_groups, dtype=torch.float64, device=tl.device)
    _check(lib.pwlq_mse_list(tl.desc, len(tl), bits, tl.mode, p.data_ptr(), m.data_ptr(),
                             out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()))
    return out


def linear_i8(xq: torch.Tensor, s_x: float, z_x: float, packed_codes: torch.Tensor,
              packed_flags: torch.Tensor, N: int, bits: int, p: torch.Tensor, m: torch.Tensor,
              want_acc: bool = False, workspace: Optional[torch.Tensor] = None, out=None):
    """pwlq_linear_i8.  xq int8 [M, K] (device); packed streams of a [N, K] weight.
    Returns (y f32 [M, N], acc i32 [3, M, N] or None)."""
    if not (xq.is_cuda and xq.dtype == torch.int8 and xq.is_contiguous() and xq.dim() == 2):
        raise ValueError("xq must be a contiguous int8 [M, K] tensor on the GPU")
    M, K = xq.shape
    if workspace is None:
        workspace = _workspace(lib.pwlq_linear_workspace_bytes(N), xq.device)
    if out is None:
        out = (torch.empty((M, N), dtype=torch.float32, device=xq.device),
               torch.empty((3, M, N), dtype=torch.int32, device=xq.device) if want_acc else None)
    y, acc = out
    _check(lib.pwlq_linear_i8(xq.data_ptr(), M, K, s_x, z_x, packed_codes.data_ptr(),
                              packed_flags.data_ptr(), N, bits, p.data_ptr(), m.data_ptr(),
                              y.data_ptr(), acc.data_ptr() if acc is not None else None,
                              workspace.data_ptr(), workspace.numel(), _stream()))
    return y, acc


def profile_enable(roles) -> None:
    """roles: False / 0 = off, True = every role, else a bit mask (bit 0 search kernel,
    bit 1 quantize kernel, bit 2 prefix-sum kernel, bit 3 inner-product kernel)."""
    lib.pwlq_profile_enable(0xF if roles is True else int(roles))


def profile_last_ms(role: int) -> float:
    return float(lib.pwlq_profile_last_ms(role))


def profile_ms(role: int, back: int) -> float:
    return float(lib.pwlq_profile_ms(role, back))


def last_search_shape():
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    lib.pwlq_last_search_shape(ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    return dict(tiles=a.value, groups=b.value, units=c.value)


def last_search_kernel() -> str:
    return lib.pwlq_last_search_kernel().decode()


def set_small_call_tiles(tiles: int) -> int:
    """Most groups a search call may have to run as one fused launch (0: never; negative:
    the default).  Returns the limit it replaces."""
    return int(lib.pwlq_set_small_call_tiles(int(tiles)))


def kernel_name(role: int) -> Optional[str]:
    s = lib.pwlq_kernel_name(role)
    return s.decode() if s else None
