"""Device-side plumbing: put a host workload into HBM and call the C ABI on it.

PyTorch is used for device allocations, copies and streams only; no tensor
arithmetic of the operator happens here.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np
import torch

from . import binding as B

_DT = {"f16": B.F16, "bf16": B.BF16}


def _to_dev(a: np.ndarray, device) -> torch.Tensor:
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


# Adapters are placed in one pool per weight kind at a stride of their size plus 64 KiB.
# With equal power-of-two sizes back to back, slice s of every adapter starts on the same
# HBM channels and the workgroups of a launch, which all read "their" slice at once, crowd a
# few channels; the offset spreads them (measured at the Llama-7B decode shape with 64
# adapters of 4 MiB: 6.5 us per add-on against 6.65 us back to back and 6.85 us with one
# allocation per adapter).
_POOL_PAD = 64 * 1024


def _pool_to_dev(arrays: List[np.ndarray], device) -> List[torch.Tensor]:
    """Copies of ``arrays`` (16-bit bit patterns) as views into one device allocation."""
    if not arrays:
        return []
    stride = (max(a.nbytes for a in arrays) + _POOL_PAD + 255) // 256 * 256
    pool = torch.empty(len(arrays) * stride, dtype=torch.uint8, device=device)
    out = []
    for i, a in enumerate(arrays):
        a = np.ascontiguousarray(a.view(np.int16) if a.dtype == np.uint16 else a)
        view = pool[i * stride:i * stride + a.nbytes].view(torch.int16).view(a.shape)
        view.copy_(torch.from_numpy(a))
        out.append(view)
    return out


class DeviceWorkload:
    """A ``sgmv_workloads.Workload`` resident on one GPU.

    ``n_sets`` independent copies of x / y are kept so that a timed loop can
    rotate over them (together with the layers) and defeat the on-die caches.
    """

    def __init__(self, w, device="cuda:0", n_sets: int = 1, max_seg_len_hint: bool = True,
                 path: int = B.PATH_AUTO, ksplit: int = 0, expand_threads: int = 0,
                 init_workspace: bool = True, max_seg_len: Optional[int] = None,
                 spin_limit: int = 0, n_proj: int = 1):
        self.w = w
        self.device = torch.device(device)
        self.A: List[torch.Tensor] = _pool_to_dev(list(w.A), self.device)
        self.B: List[torch.Tensor] = _pool_to_dev(list(w.B), self.device)
        a_ptrs = [0 if a < 0 else self.A[a].data_ptr() for a in w.seg_adapter]
        b_ptrs = [0 if a < 0 else self.B[a].data_ptr() for a in w.seg_adapter]
        self.A_ptrs = torch.tensor(a_ptrs, dtype=torch.int64, device=self.device)
        self.B_ptrs = torch.tensor(b_ptrs, dtype=torch.int64, device=self.device)
        self.seg_starts = _to_dev(w.seg_starts.astype(np.int32), self.device)
        self.x = [_to_dev(w.x, self.device) for _ in range(n_sets)]
        self.y0 = _to_dev(w.y0, self.device)
        self.y = [self.y0.clone() for _ in range(n_sets)]
        # n_proj > 1: room for multi-projection calls that share the shrink's pass over x
        self.ws_bytes = max(B.sgmv_workspace_bytes_multi(w.n_tokens, w.r, n_proj), 256)
        # deliberately not zero-filled by torch: sgmv_workspace_init does that
        self.workspace = torch.full((self.ws_bytes,), 0xA5, dtype=torch.uint8, device=self.device)
        if init_workspace:
            B.sgmv_workspace_init(self.workspace, self.ws_bytes)
            torch.cuda.synchronize(self.device)   # later calls may use other streams
        self.problem = B.make_problem(
            _DT[w.dtype], w.h_in, w.h_out, w.r, w.num_layers, w.n_tokens,
            workspace=self.workspace, workspace_bytes=self.ws_bytes,
            max_seg_len=(max_seg_len if max_seg_len is not None else
                         w.max_seg_len if max_seg_len_hint else 0), path=path, ksplit=ksplit,
            expand_threads=expand_threads, workspace_ready=1 if init_workspace else 0,
            spin_limit=spin_limit)

    # -- the three entry points, on set `k` ---------------------------------
    def add_lora(self, layer_idx: int = 0, k: int = 0, stream=None, scale: Optional[float] = None):
        return B.sgmv_add_lora(self.problem, self.y[k], self.x[k], self.A_ptrs, self.B_ptrs,
                               self.seg_starts, self.w.n_segs, layer_idx,
                               self.w.scale if scale is None else scale, stream)

    def shrink(self, v: torch.Tensor, layer_idx: int = 0, k: int = 0, stream=None):
        return B.sgmv_shrink(self.problem, v, self.x[k], self.A_ptrs, self.seg_starts,
                             self.w.n_segs, layer_idx, stream)

    def expand(self, v: torch.Tensor, layer_idx: int = 0, k: int = 0, stream=None,
               scale: Optional[float] = None):
        return B.sgmv_expand(self.problem, self.y[k], v, self.B_ptrs, self.seg_starts,
                             self.w.n_segs, layer_idx, self.w.scale if scale is None else scale,
                             stream)

    def check(self, stream=None) -> int:
        """Synchronous health check of the workspace (0 = fine)."""
        return B.sgmv_workspace_check(self.workspace, stream)

    def reset_y(self, k: Optional[int] = None):
        for i in (range(len(self.y)) if k is None else [k]):
            self.y[i].copy_(self.y0)

    def y_bits(self, k: int = 0) -> np.ndarray:
        torch.cuda.synchronize(self.device)
        return self.y[k].cpu().numpy().view(np.uint16)
