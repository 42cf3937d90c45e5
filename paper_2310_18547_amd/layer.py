"""The seven LoRA add-ons of one decoder layer (call plumbing only).

The paper applies LoRA to every dense projection of a transformer layer -- query, key,
value, output, gate, up, down -- and builds the segment indices once per model invocation,
so one ``seg_starts`` serves all of them (Background, "Low-Rank Adaptation"; the remark on
segment indices in the section on the runner).  ``LoraLayer`` issues those seven add-ons
through the C ABI: the projections that read the same activations (q/k/v, gate/up) go into
one ``sgmv_add_lora_multi`` call each, o and down are single ``sgmv_add_lora`` calls.  All
calls share one workspace and must be enqueued on one stream.
"""
from __future__ import annotations

from typing import Dict, Sequence

import torch

from . import binding as B

PROJECTIONS = ("q", "k", "v", "o", "gate", "up", "down")
GROUPS = (("q", "k", "v"), ("o",), ("gate", "up"), ("down",))


def projection_shapes(h: int, ffn: int) -> Dict[str, tuple]:
    """name -> (h_in, h_out) of a Llama-style decoder layer."""
    return {"q": (h, h), "k": (h, h), "v": (h, h), "o": (h, h), "gate": (h, ffn), "up": (h, ffn),
            "down": (ffn, h)}


class LoraLayer:
    def __init__(self, h: int, ffn: int, r: int, num_layers: int, n_tokens: int, dtype: int,
                 A_ptrs: Dict[str, torch.Tensor], B_ptrs: Dict[str, torch.Tensor],
                 seg_starts: torch.Tensor, n_segs: int, max_seg_len: int, device="cuda:0"):
        self.shapes = projection_shapes(h, ffn)
        self.A_ptrs, self.B_ptrs = A_ptrs, B_ptrs
        self.seg_starts, self.n_segs = seg_starts, n_segs
        self.ws_bytes = max(B.sgmv_workspace_bytes(n_tokens, r), 256)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        B.sgmv_workspace_init(self.workspace, self.ws_bytes)
        torch.cuda.synchronize(device)
        self.problem = {n: B.make_problem(dtype, i, o, r, num_layers, n_tokens,
                                          workspace=self.workspace, workspace_bytes=self.ws_bytes,
                                          max_seg_len=max_seg_len, workspace_ready=1)
                        for n, (i, o) in self.shapes.items()}

    def add_lora(self, name: str, y, x, layer_idx: int, scale: float = 1.0, stream=None):
        return B.sgmv_add_lora(self.problem[name], y, x, self.A_ptrs[name], self.B_ptrs[name],
                               self.seg_starts, self.n_segs, layer_idx, scale, stream)

    def add_lora_group(self, names: Sequence[str], ys, xs, layer_idx: int, scale: float = 1.0,
                       stream=None):
        """Projections of one shape in one call (``ys`` / ``xs`` in the order of ``names``)."""
        if len(names) == 1:
            return self.add_lora(names[0], ys[0], xs[0], layer_idx, scale, stream)
        return B.sgmv_add_lora_multi(self.problem[names[0]], list(ys), list(xs),
                                     [self.A_ptrs[n] for n in names],
                                     [self.B_ptrs[n] for n in names], self.seg_starts,
                                     self.n_segs, layer_idx, scale, stream)

    def check(self, stream=None) -> int:
        return B.sgmv_workspace_check(self.workspace, stream)
