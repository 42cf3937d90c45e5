"""On-demand loading of LoRA adapters next to running SGMV calls (device plumbing only).

The paper loads an adapter's weights from host memory when the first request for it
arrives, with an asynchronous host-to-device copy that overlaps the batch that is running,
and the adapter joins the batch at the next step (section "On-demand loading of LoRA
models").  With this library an adapter is "in the batch" when its device pointers stand in
the ``A_ptrs`` / ``B_ptrs`` arrays, so loading one is: copy on a second stream, record an
event, make the compute stream wait for it, write two pointers.  The library itself keeps no
adapter state and no kernel is involved; PyTorch provides memory, streams and events.
"""
from __future__ import annotations

from typing import List, Tuple

import torch

_POOL_PAD = 64 * 1024     # slots are staggered like device.py's pools (HBM channel spread)


class AdapterPool:
    """``n_slots`` device slots for the weights of one projection:
    A ``[num_layers][h_in][r]`` and B ``[num_layers][r][h_out]``, 16-bit bit patterns."""

    def __init__(self, n_slots: int, num_layers: int, h_in: int, h_out: int, r: int,
                 device="cuda:0"):
        self.device = torch.device(device)
        self.shape_A = (num_layers, h_in, r)
        self.shape_B = (num_layers, r, h_out)
        self.n_slots = n_slots

        def pool(shape) -> List[torch.Tensor]:
            size = 2 * shape[0] * shape[1] * shape[2]
            stride = (size + _POOL_PAD + 255) // 256 * 256
            buf = torch.empty(n_slots * stride, dtype=torch.uint8, device=self.device)
            return [buf[i * stride:i * stride + size].view(torch.int16).view(shape)
                    for i in range(n_slots)]

        self.A = pool(self.shape_A)
        self.B = pool(self.shape_B)
        # pinned staging for the two pointers a bind writes (one pair per slot, kept alive here)
        self._ptr_host = [torch.tensor([self.A[i].data_ptr(), self.B[i].data_ptr()],
                                       dtype=torch.int64).pin_memory() for i in range(n_slots)]

    @staticmethod
    def pin(bits) -> torch.Tensor:
        """A pinned host copy of a numpy array of 16-bit patterns."""
        import numpy as np
        a = np.ascontiguousarray(bits.view(np.int16) if bits.dtype == np.uint16 else bits)
        t = torch.empty(a.shape, dtype=torch.int16, pin_memory=True)
        t.copy_(torch.from_numpy(a))
        return t

    def pointers(self, slot: int) -> Tuple[int, int]:
        return self.A[slot].data_ptr(), self.B[slot].data_ptr()

    def load_async(self, slot: int, host_A: torch.Tensor, host_B: torch.Tensor,
                   copy_stream: torch.cuda.Stream) -> torch.cuda.Event:
        """Start copying pinned host weights into ``slot`` on ``copy_stream``; returns the
        event that marks the end of the copy.  The slot must not be in use by a running or
        queued call."""
        assert host_A.is_pinned() and host_B.is_pinned(), "on-demand loads need pinned host memory"
        assert tuple(host_A.shape) == self.shape_A and tuple(host_B.shape) == self.shape_B
        with torch.cuda.stream(copy_stream):
            self.A[slot].copy_(host_A, non_blocking=True)
            self.B[slot].copy_(host_B, non_blocking=True)
            ev = torch.cuda.Event()
            ev.record(copy_stream)
        return ev

    def bind(self, A_ptrs: torch.Tensor, B_ptrs: torch.Tensor, seg: int, slot: int,
             compute_stream: torch.cuda.Stream, ready: torch.cuda.Event) -> None:
        """Make segment ``seg`` of the pointer arrays use ``slot`` for every call enqueued on
        ``compute_stream`` after this: the stream waits for the copy, then the two pointers
        are written in stream order (calls already queued keep the old adapter)."""
        compute_stream.wait_event(ready)
        with torch.cuda.stream(compute_stream):
            A_ptrs[seg:seg + 1].copy_(self._ptr_host[slot][0:1], non_blocking=True)
            B_ptrs[seg:seg + 1].copy_(self._ptr_host[slot][1:2], non_blocking=True)
