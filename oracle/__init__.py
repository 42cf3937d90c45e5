"""CPU oracle for SGMV -- TEST INFRASTRUCTURE, not part of the product path.

Thin ctypes access to ``sgmv_oracle.c`` (plain C, compiled with gcc).  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library never does.  Nothing here imports the GPU package.

All tensors are host ``numpy`` arrays; 16-bit tensors are ``uint16`` bit
patterns together with a dtype tag ("f16" / "bf16").
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sgmv_oracle.c")
_LIB = os.path.join(_HERE, "libsgmv_oracle.so")
_DT = {"f16": 0, "bf16": 1}
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared",
                               "-ffp-contract=off", "-fno-fast-math", "-pthread",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c = ctypes
        L.sgmv_oracle_shrink.argtypes = [c.c_int, c.c_int, c.c_int, c.c_void_p, c.c_void_p,
                                         c.c_void_p, c.c_void_p, c.c_int, c.c_int, c.c_int, c.c_int]
        L.sgmv_oracle_expand.argtypes = [c.c_int, c.c_int, c.c_int, c.c_void_p, c.c_void_p,
                                         c.c_void_p, c.c_void_p, c.c_int, c.c_int, c.c_float,
                                         c.c_int, c.c_int]
        L.sgmv_oracle_add_lora.argtypes = [c.c_int, c.c_int, c.c_int, c.c_int, c.c_void_p,
                                           c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                           c.c_int, c.c_int, c.c_float, c.c_int, c.c_int]
        for f in (L.sgmv_oracle_shrink, L.sgmv_oracle_expand, L.sgmv_oracle_add_lora):
            f.restype = c.c_int
        L.sgmv_oracle_decode.argtypes = [c.c_int, c.c_void_p, c.c_void_p, c.c_size_t]
        L.sgmv_oracle_encode.argtypes = [c.c_int, c.c_void_p, c.c_void_p, c.c_size_t]
        L.sgmv_oracle_decode.restype = None
        L.sgmv_oracle_encode.restype = None
        _lib = L
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def _check16(a, shape=None):
    assert a.dtype == np.uint16 and a.flags.c_contiguous, "expected contiguous uint16 bits"
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)


def pointer_array(mats: Sequence[Optional[np.ndarray]]) -> np.ndarray:
    """Host array of host addresses, one per segment; ``None`` becomes NULL."""
    out = np.zeros(len(mats), np.uint64)
    for i, m in enumerate(mats):
        if m is not None:
            _check16(m)
            out[i] = m.ctypes.data
    return out


def decode(bits: np.ndarray, dtype: str) -> np.ndarray:
    _check16(bits)
    out = np.empty(bits.shape, np.float32)
    _load().sgmv_oracle_decode(_DT[dtype], bits.ctypes.data, out.ctypes.data, bits.size)
    return out


def encode(vals: np.ndarray, dtype: str) -> np.ndarray:
    vals = np.ascontiguousarray(vals, np.float32)
    out = np.empty(vals.shape, np.uint16)
    _load().sgmv_oracle_encode(_DT[dtype], vals.ctypes.data, out.ctypes.data, vals.size)
    return out


def shrink(dtype, v, x, A_list, seg_starts, layer_idx=0, acc64=False, n_threads=1):
    """In place: v[rows of seg i] += x[rows of seg i] @ A_list[i][layer_idx]."""
    seg_starts = np.ascontiguousarray(seg_starts, np.int32)
    n = len(seg_starts) - 1
    assert len(A_list) == n
    T, h_in = x.shape
    _check16(x)
    assert v.dtype == np.float32 and v.flags.c_contiguous and v.shape[0] == T
    r = v.shape[1]
    for m in A_list:
        if m is not None:
            assert m.ndim == 3 and m.shape[1:] == (h_in, r) and 0 <= layer_idx < m.shape[0]
    ptrs = pointer_array(A_list)
    rc = _load().sgmv_oracle_shrink(_DT[dtype], h_in, r, v.ctypes.data, x.ctypes.data,
                                    ptrs.ctypes.data, seg_starts.ctypes.data, n, layer_idx,
                                    int(acc64), n_threads)
    assert rc == 0
    return v


def expand(dtype, y, v, B_list, seg_starts, layer_idx=0, scale=1.0, acc64=False, n_threads=1):
    """In place: y[rows of seg i] += scale * v[rows] @ B_list[i][layer_idx]."""
    seg_starts = np.ascontiguousarray(seg_starts, np.int32)
    n = len(seg_starts) - 1
    assert len(B_list) == n
    T, h_out = y.shape
    _check16(y)
    assert v.dtype == np.float32 and v.flags.c_contiguous and v.shape[0] == T
    r = v.shape[1]
    for m in B_list:
        if m is not None:
            assert m.ndim == 3 and m.shape[1:] == (r, h_out) and 0 <= layer_idx < m.shape[0]
    ptrs = pointer_array(B_list)
    rc = _load().sgmv_oracle_expand(_DT[dtype], r, h_out, y.ctypes.data, v.ctypes.data,
                                    ptrs.ctypes.data, seg_starts.ctypes.data, n, layer_idx,
                                    float(scale), int(acc64), n_threads)
    assert rc == 0
    return y


def add_lora(dtype, y, x, A_list, B_list, seg_starts, layer_idx=0, scale=1.0,
             acc64=False, n_threads=1):
    """In place: y[rows of seg i] += scale * (x[rows] @ A_i[layer]) @ B_i[layer]."""
    seg_starts = np.ascontiguousarray(seg_starts, np.int32)
    n = len(seg_starts) - 1
    assert len(A_list) == n and len(B_list) == n
    T, h_in = x.shape
    T2, h_out = y.shape
    assert T == T2
    _check16(x)
    _check16(y)
    r = None
    for a, b in zip(A_list, B_list):
        if a is not None and b is not None:
            r = a.shape[2]
            assert a.shape[1:] == (h_in, r) and b.shape[1:] == (r, h_out)
            assert 0 <= layer_idx < a.shape[0] and a.shape[0] == b.shape[0]
    if r is None:
        return y
    pa, pb = pointer_array(A_list), pointer_array(B_list)
    rc = _load().sgmv_oracle_add_lora(_DT[dtype], h_in, h_out, r, y.ctypes.data, x.ctypes.data,
                                      pa.ctypes.data, pb.ctypes.data, seg_starts.ctypes.data,
                                      n, layer_idx, float(scale), int(acc64), n_threads)
    assert rc == 0
    return y


def run_workload(w, op="add_lora", layer_idx=0, acc64=False, n_threads=1, v=None):
    """Convenience: run one operator on a ``sgmv_workloads.Workload``.

    Returns y (uint16 bits) for "add_lora"/"expand", v (fp32) for "shrink".
    """
    A_list = [None if a < 0 else w.A[a] for a in w.seg_adapter]
    B_list = [None if a < 0 else w.B[a] for a in w.seg_adapter]
    if op == "add_lora":
        y = w.y0.copy()
        return add_lora(w.dtype, y, w.x, A_list, B_list, w.seg_starts, layer_idx, w.scale,
                        acc64, n_threads)
    if op == "shrink":
        vv = np.zeros((w.n_tokens, w.r), np.float32) if v is None else v.copy()
        return shrink(w.dtype, vv, w.x, A_list, w.seg_starts, layer_idx, acc64, n_threads)
    if op == "expand":
        assert v is not None
        y = w.y0.copy()
        return expand(w.dtype, y, v, B_list, w.seg_starts, layer_idx, w.scale, acc64, n_threads)
    raise ValueError(op)
