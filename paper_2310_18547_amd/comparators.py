"""The paper's two comparison implementations of the batched LoRA add-on, on the same GPU.

These are NOT part of the SGMV path: they are library comparators (PyTorch tensor ops on
ROCm, i.e. rocBLAS / hipBLASLt GEMMs) used by ``bench.py --compare`` to reproduce the shape of
the paper's LoRA-operator microbenchmark (section "Microbenchmarks", LoRA operator figure):

* **Loop**: a for-loop over the LoRA models of the batch, two small GEMMs per model.
* **Gather-BMM**: gather every token's weights into ``[tokens, h_in, r]`` / ``[tokens, r, h_out]``
  stacks, then two batched matrix multiplications.  The gather moves
  ``tokens * (h_in * r + r * h_out) * 2`` bytes of weights on top of what SGMV reads
  (the paper's remark on Gather-BMM's extra I/O).

Both compute ``y[rows of segment i] += scale * (x[rows] @ A_i) @ B_i`` with 16-bit
storage; the intermediate is kept in the 16-bit type as a plain PyTorch user would.
"""
from __future__ import annotations

from typing import List, Sequence

import torch


def _typed(t: torch.Tensor, dtype: str) -> torch.Tensor:
    """Reinterpret an int16 bit-pattern tensor as fp16 / bf16 (no copy)."""
    return t.view(torch.float16 if dtype == "f16" else torch.bfloat16)


class Comparators:
    """Loop and Gather-BMM over a ``DeviceWorkload``'s device tensors."""

    def __init__(self, d):
        w = d.w
        self.d, self.w = d, w
        self.A = [_typed(a, w.dtype) for a in d.A]          # [L, h_in, r] per adapter
        self.B = [_typed(b, w.dtype) for b in d.B]          # [L, r, h_out] per adapter
        self.x = [_typed(x, w.dtype) for x in d.x]
        self.y = [_typed(y, w.dtype) for y in d.y]
        starts = [int(v) for v in w.seg_starts]
        self.segs = [(starts[i], starts[i + 1], int(w.seg_adapter[i])) for i in range(w.n_segs)
                     if starts[i + 1] > starts[i] and w.seg_adapter[i] >= 0]
        # adapter id of every token, for the gather
        tok = torch.full((w.n_tokens,), -1, dtype=torch.int64)
        for lo, hi, a in self.segs:
            tok[lo:hi] = a
        self.rows = torch.nonzero(tok >= 0).flatten().to(d.device)
        self.tok_adapter = tok[tok >= 0].to(d.device)
        self.A_all = None
        self.B_all = None

    def loop(self, layer: int, k: int = 0) -> None:
        x, y, s = self.x[k], self.y[k], self.w.scale
        for lo, hi, a in self.segs:
            v = x[lo:hi] @ self.A[a][layer]
            y[lo:hi] += s * (v @ self.B[a][layer]) if s != 1.0 else v @ self.B[a][layer]

    def _stacks(self):
        if self.A_all is None:      # [adapters, L, h_in, r]: the pool the gather indexes into
            self.A_all = torch.stack(self.A)
            self.B_all = torch.stack(self.B)
        return self.A_all, self.B_all

    def gather_bmm(self, layer: int, k: int = 0) -> None:
        A_all, B_all = self._stacks()
        x, y, s = self.x[k], self.y[k], self.w.scale
        Ag = A_all[self.tok_adapter, layer]                  # gather: [T, h_in, r]
        Bg = B_all[self.tok_adapter, layer]                  # gather: [T, r, h_out]
        v = torch.bmm(x[self.rows].unsqueeze(1), Ag)         # [T, 1, r]
        out = torch.bmm(v, Bg).squeeze(1)                    # [T, h_out]
        y[self.rows] += s * out if s != 1.0 else out
