"""ctypes binding of include/sgmv.h.

The functions have the C names and the C argument order.  Pointer arguments
accept a ``torch`` tensor (its ``data_ptr()`` is taken), an ``int`` address or
``None``; nothing is copied, converted or computed here.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
# SGMV_LIBRARY names another build of the same sources in this directory (the tuning build
# with the in-kernel timeline, libsgmv_trace.so); the default is the library proper
_LIB_PATH = os.path.join(_HERE, os.path.basename(os.environ.get("SGMV_LIBRARY", "libsgmv.so")))

F16, BF16 = 0, 1
PATH_AUTO, PATH_VECTOR, PATH_MATRIX, PATH_FUSED, PATH_WHOLE, PATH_ROWS = 0, 1, 2, 3, 4, 5


class SgmvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({sgmv_status_string(status)})")


class SgmvProblem(ctypes.Structure):
    """Mirror of ``struct sgmv_problem``."""
    _fields_ = [
        ("dtype", ctypes.c_int32),
        ("h_in", ctypes.c_int32),
        ("h_out", ctypes.c_int32),
        ("r", ctypes.c_int32),
        ("num_layers", ctypes.c_int32),
        ("n_tokens", ctypes.c_int32),
        ("max_seg_len", ctypes.c_int32),
        ("path", ctypes.c_int32),
        ("ksplit", ctypes.c_int32),
        ("expand_threads", ctypes.c_int32),
        ("workspace_ready", ctypes.c_int32),
        ("spin_limit", ctypes.c_int32),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
    ]


def library_path() -> str:
    return _LIB_PATH


class SgmvPlan(ctypes.Structure):
    """Mirror of ``struct sgmv_plan``."""
    _fields_ = [
        ("kernel", ctypes.c_int32),
        ("launches", ctypes.c_int32),
        ("slices", ctypes.c_int32),
        ("workgroups", ctypes.c_int32),
        ("lds_bytes", ctypes.c_int32),
        ("reserved", ctypes.c_int32 * 3),
    ]


KERNEL_NONE, KERNEL_FUSED, KERNEL_TILE, KERNEL_MULTI_SIDE, KERNEL_MULTI_PIPELINED, KERNEL_VECTOR, \
    KERNEL_MATRIX, KERNEL_SEQUENCE, KERNEL_WHOLE = range(9)
KERNEL_NAMES = {KERNEL_NONE: "none", KERNEL_FUSED: "fused", KERNEL_TILE: "tile",
                KERNEL_MULTI_SIDE: "multi_side", KERNEL_MULTI_PIPELINED: "multi_pipelined",
                KERNEL_VECTOR: "vector", KERNEL_MATRIX: "matrix", KERNEL_WHOLE: "whole"}


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2310_18547_amd.build` "
            "(there is no fallback implementation)")
    L = ctypes.CDLL(_LIB_PATH)
    c = ctypes
    P = c.POINTER(SgmvProblem)
    L.sgmv_status_string.argtypes = [c.c_int]
    L.sgmv_status_string.restype = c.c_char_p
    L.sgmv_workspace_bytes.argtypes = [c.c_int32, c.c_int32]
    L.sgmv_workspace_bytes.restype = c.c_size_t
    L.sgmv_workspace_bytes_multi.argtypes = [c.c_int32, c.c_int32, c.c_int32]
    L.sgmv_workspace_bytes_multi.restype = c.c_size_t
    L.sgmv_workspace_init.argtypes = [c.c_void_p, c.c_size_t, c.c_void_p]
    L.sgmv_workspace_init.restype = c.c_int
    L.sgmv_workspace_check.argtypes = [c.c_void_p, c.c_void_p]
    L.sgmv_workspace_check.restype = c.c_int
    L.sgmv_validate_segments.argtypes = [c.c_void_p, c.c_int32, c.c_int32]
    L.sgmv_validate_segments.restype = c.c_int
    L.sgmv_shrink.argtypes = [P, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32,
                              c.c_int32, c.c_void_p]
    L.sgmv_shrink.restype = c.c_int
    L.sgmv_expand.argtypes = [P, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32,
                              c.c_int32, c.c_float, c.c_void_p]
    L.sgmv_expand.restype = c.c_int
    L.sgmv_add_lora.argtypes = [P, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                c.c_int32, c.c_int32, c.c_float, c.c_void_p]
    L.sgmv_add_lora.restype = c.c_int
    L.sgmv_add_lora_static.argtypes = L.sgmv_add_lora.argtypes
    L.sgmv_add_lora_static.restype = c.c_int
    L.sgmv_add_lora_multi.argtypes = [P, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                      c.c_void_p, c.c_int32, c.c_int32, c.c_float, c.c_void_p]
    L.sgmv_add_lora_multi.restype = c.c_int
    L.sgmv_probe.argtypes = [c.c_int, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    L.sgmv_probe.restype = c.c_int
    L.sgmv_plan_add_lora.argtypes = [P, c.c_int32, c.c_int32, c.POINTER(SgmvPlan)]
    L.sgmv_plan_add_lora.restype = c.c_int
    L.sgmv_plan_shrink.argtypes = [P, c.c_int32, c.POINTER(SgmvPlan)]
    L.sgmv_plan_shrink.restype = c.c_int
    L.sgmv_plan_expand.argtypes = [P, c.c_int32, c.POINTER(SgmvPlan)]
    L.sgmv_plan_expand.restype = c.c_int
    return L


lib = _load()


def _addr(a) -> Optional[int]:
    if a is None:
        return None
    if isinstance(a, int):
        return a
    if hasattr(a, "data_ptr"):
        return a.data_ptr()
    if hasattr(a, "ctypes"):          # host numpy array (sgmv_validate_segments only)
        return a.ctypes.data
    raise TypeError(f"cannot take the address of {type(a)!r}")


def _stream(s) -> Optional[int]:
    if s is None or isinstance(s, int):
        return s
    return s.cuda_stream              # a torch.cuda.Stream


def make_problem(dtype: int, h_in: int, h_out: int, r: int, num_layers: int, n_tokens: int,
                 workspace=None, workspace_bytes: int = 0, max_seg_len: int = 0,
                 path: int = PATH_AUTO, ksplit: int = 0, expand_threads: int = 0,
                 workspace_ready: int = 0, spin_limit: int = 0) -> SgmvProblem:
    return SgmvProblem(dtype, h_in, h_out, r, num_layers, n_tokens, max_seg_len, path, ksplit,
                       expand_threads, workspace_ready, spin_limit, _addr(workspace), workspace_bytes)


def sgmv_status_string(status: int) -> str:
    return lib.sgmv_status_string(int(status)).decode()


def sgmv_workspace_bytes(n_tokens: int, r: int) -> int:
    return int(lib.sgmv_workspace_bytes(n_tokens, r))


def sgmv_workspace_bytes_multi(n_tokens: int, r: int, n_proj: int) -> int:
    return int(lib.sgmv_workspace_bytes_multi(n_tokens, r, n_proj))


def sgmv_workspace_init(workspace, workspace_bytes: int, stream=None, check: bool = True) -> int:
    rc = lib.sgmv_workspace_init(_addr(workspace), workspace_bytes, _stream(stream))
    if check and rc != 0:
        raise SgmvError(rc, "sgmv_workspace_init")
    return rc


def sgmv_workspace_check(workspace, stream=None) -> int:
    return lib.sgmv_workspace_check(_addr(workspace), _stream(stream))


def sgmv_validate_segments(host_seg_starts, n_segs: int, n_tokens: int) -> int:
    return lib.sgmv_validate_segments(_addr(host_seg_starts), n_segs, n_tokens)


def sgmv_shrink(p: SgmvProblem, v, x, A_ptrs, seg_starts, n_segs: int, layer_idx: int,
                stream=None, check: bool = True) -> int:
    rc = lib.sgmv_shrink(ctypes.byref(p), _addr(v), _addr(x), _addr(A_ptrs), _addr(seg_starts),
                         n_segs, layer_idx, _stream(stream))
    if check and rc != 0:
        raise SgmvError(rc, "sgmv_shrink")
    return rc


def sgmv_expand(p: SgmvProblem, y, v, B_ptrs, seg_starts, n_segs: int, layer_idx: int,
                scale: float, stream=None, check: bool = True) -> int:
    rc = lib.sgmv_expand(ctypes.byref(p), _addr(y), _addr(v), _addr(B_ptrs), _addr(seg_starts),
                         n_segs, layer_idx, scale, _stream(stream))
    if check and rc != 0:
        raise SgmvError(rc, "sgmv_expand")
    return rc


def sgmv_add_lora(p: SgmvProblem, y, x, A_ptrs, B_ptrs, seg_starts, n_segs: int, layer_idx: int,
                  scale: float, stream=None, check: bool = True) -> int:
    rc = lib.sgmv_add_lora(ctypes.byref(p), _addr(y), _addr(x), _addr(A_ptrs), _addr(B_ptrs),
                           _addr(seg_starts), n_segs, layer_idx, scale, _stream(stream))
    if check and rc != 0:
        raise SgmvError(rc, "sgmv_add_lora")
    return rc


def sgmv_add_lora_static(p: SgmvProblem, y, x, A_ptrs, B_ptrs, seg_starts, n_segs: int,
                         layer_idx: int, scale: float, stream=None, check: bool = True) -> int:
    rc = lib.sgmv_add_lora_static(ctypes.byref(p), _addr(y), _addr(x), _addr(A_ptrs), _addr(B_ptrs),
                                  _addr(seg_starts), n_segs, layer_idx, scale, _stream(stream))
    if check and rc != 0:
        raise SgmvError(rc, "sgmv_add_lora_static")
    return rc


STATIC_SCRATCH_BYTES = 9 << 20
STATIC_MAX_WORKSPACE_BYTES = 8 << 20


def sgmv_add_lora_multi(p: SgmvProblem, ys, xs, A_ptrs, B_ptrs, seg_starts, n_segs: int,
                        layer_idx: int, scale: float, stream=None, check: bool = True) -> int:
    """``ys, xs, A_ptrs, B_ptrs`` are sequences of equal length (one entry per add-on)."""
    n = len(ys)
    arr = ctypes.c_void_p * n
    rc = lib.sgmv_add_lora_multi(
        ctypes.byref(p), n, arr(*[_addr(a) for a in ys]), arr(*[_addr(a) for a in xs]),
        arr(*[_addr(a) for a in A_ptrs]), arr(*[_addr(a) for a in B_ptrs]), _addr(seg_starts),
        n_segs, layer_idx, scale, _stream(stream))
    if check and rc != 0:
        raise SgmvError(rc, "sgmv_add_lora_multi")
    return rc


def sgmv_plan_expand(p: SgmvProblem, n_segs: int, check: bool = True):
    """Host-only: the ``SgmvPlan`` of a stand-alone ``sgmv_expand`` (``check=False``: ``(status, plan)``)."""
    plan = SgmvPlan()
    rc = lib.sgmv_plan_expand(ctypes.byref(p), n_segs, ctypes.byref(plan))
    if not check:
        return rc, plan
    if rc != 0:
        raise SgmvError(rc, "sgmv_plan_expand")
    return plan


def sgmv_plan_shrink(p: SgmvProblem, n_segs: int, check: bool = True):
    """Host-only: the ``SgmvPlan`` of a stand-alone ``sgmv_shrink`` (``check=False``: ``(status, plan)``)."""
    plan = SgmvPlan()
    rc = lib.sgmv_plan_shrink(ctypes.byref(p), n_segs, ctypes.byref(plan))
    if not check:
        return rc, plan
    if rc != 0:
        raise SgmvError(rc, "sgmv_plan_shrink")
    return plan


PROBE_EMPTY, PROBE_READ, PROBE_COPY, PROBE_HANDOFF = 0, 1, 2, 3


def sgmv_probe(kind: int, src=None, dst=None, nbytes: int = 0, stream=None, check: bool = True) -> int:
    rc = lib.sgmv_probe(kind, _addr(src), _addr(dst), nbytes, _stream(stream))
    if check and rc != 0:
        raise SgmvError(rc, "sgmv_probe")
    return rc


def sgmv_plan_add_lora(p: SgmvProblem, n_segs: int, n_proj: int = 1, check: bool = True):
    """Host-only: the ``SgmvPlan`` of the call (``check=False``: ``(status, plan)``)."""
    plan = SgmvPlan()
    rc = lib.sgmv_plan_add_lora(ctypes.byref(p), n_segs, n_proj, ctypes.byref(plan))
    if not check:
        return rc, plan
    if rc != 0:
        raise SgmvError(rc, "sgmv_plan_add_lora")
    return plan
