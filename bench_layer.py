#!/usr/bin/env python3
"""Transformer-layer microbenchmark: what the LoRA add-ons cost next to the dense projections.

    python bench_layer.py [--model 7b|13b] [--batch 64] [--seq 1] [--rank 16] [--steps 200]

One *step* is the seven dense projections of one decoder layer (attention itself is left out) with a
Distinct batch: every request has its own LoRA adapter on all seven projections.  ``--seq 1`` is the
decode shape (one token per request); ``--seq 512`` / ``2048`` are the prefill shapes of the paper's
transformer-layer benchmark: every request contributes a segment of that many rows (the paper
applies LoRA to q, k, v, o, gate, up, down); ``--mix uniform|skewed|identical`` makes the decode
batch share adapters the way the operator microbenchmark's popularity mixes do.  The
backbone GEMMs are library calls (PyTorch matmul = rocBLAS / hipBLASLt); the add-ons are this
library's kernels, issued three ways:

* ``backbone``        the seven GEMMs alone;
* ``lora_single``     + seven ``sgmv_add_lora`` calls;
* ``lora_multi``      + ``sgmv_add_lora_multi`` for q/k/v and for gate/up, single calls for o, down.

Consecutive steps cycle over ``--layers`` sets of backbone and adapter weights so that nothing
is served from the on-die caches.  Everything is synthetic (random weights, as in the paper's
microbenchmarks).  Prints ONE JSON line.  This follows the paper's transformer-layer
benchmark in spirit only: no attention kernel, one GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MODELS = {"7b": (4096, 11008), "13b": (5120, 13824)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", choices=sorted(MODELS), default="7b")
    ap.add_argument("--batch", type=int, default=64, help="requests, each with its own adapter")
    ap.add_argument("--seq", type=int, default=1, help="token rows per request (1 = decode)")
    ap.add_argument("--mix", choices=["distinct", "uniform", "skewed", "identical"], default="distinct",
                    help="adapter popularity over the --batch decode rows (the operator microbenchmark's mixes): "
                         "rows that share an adapter form one segment")
    ap.add_argument("--rank", type=int, default=16)
    ap.add_argument("--layers", type=int, default=4, help="weight sets cycled through")
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--blocks", type=int, default=3)
    args = ap.parse_args()

    import numpy as np
    import torch
    from paper_2310_18547_amd import binding as B

    assert torch.cuda.is_available(), "bench_layer.py needs a GPU"
    dev = torch.device("cuda:0")
    h, ffn = MODELS[args.model]
    n_req, r, L = args.batch, args.rank, args.layers
    T = n_req * args.seq  # token rows: request i owns rows i * seq .. (i + 1) * seq - 1
    seg_lens = [args.seq] * n_req
    if args.mix != "distinct":
        # decode rows of requests that share adapters: segments as the seeded workload generator draws them
        assert args.seq == 1, "--mix describes a decode batch"
        import sgmv_workloads as wl
        starts = wl.popularity(args.mix, batch=args.batch, h_in=64, h_out=64, r=8, num_layers=1, seed=0).seg_starts
        seg_lens = np.diff(starts).tolist()
        n_req = len(seg_lens)  # adapters in the batch
    gen = torch.Generator(device=dev).manual_seed(0)
    f16 = torch.float16

    def rnd(*shape, std=1.0):
        return (torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32) * std).to(f16)

    # projections: name -> (h_in, h_out)
    shapes = {"q": (h, h), "k": (h, h), "v": (h, h), "o": (h, h), "gate": (h, ffn), "up": (h, ffn),
              "down": (ffn, h)}
    W = {n: [rnd(i, o, std=i ** -0.5) for _ in range(L)] for n, (i, o) in shapes.items()}
    # adapters: one per request and projection, stacked over the cycled layers
    def pool(count, shape, std):
        # one allocation per weight kind, adapter i at i * (size + 64 KiB): equal power-of-two
        # sizes back to back would start every adapter's slices on the same HBM channels
        size = 2
        for d in shape:
            size *= d
        stride = (size + 65536 + 255) // 256 * 256
        buf = torch.empty(count * stride, dtype=torch.uint8, device=dev)
        views = [buf[k * stride:k * stride + size].view(f16).view(*shape) for k in range(count)]
        for v in views:
            v.copy_(rnd(*shape, std=std))
        return views

    A = {n: pool(n_req, (L, i, r), i ** -0.5) for n, (i, o) in shapes.items()}
    Bw = {n: pool(n_req, (L, r, o), r ** -0.5) for n, (i, o) in shapes.items()}
    A_ptrs = {n: torch.tensor([t.data_ptr() for t in A[n]], dtype=torch.int64, device=dev) for n in shapes}
    B_ptrs = {n: torch.tensor([t.data_ptr() for t in Bw[n]], dtype=torch.int64, device=dev) for n in shapes}
    seg_starts = torch.tensor(np.concatenate(([0], np.cumsum(seg_lens))), dtype=torch.int32, device=dev)
    x = rnd(T, h)
    y = {n: torch.empty(T, o, dtype=f16, device=dev) for n, (i, o) in shapes.items()}

    ws_bytes = B.sgmv_workspace_bytes_multi(T, r, 3)  # q / k / v in one call may share the pass over x
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    B.sgmv_workspace_init(ws, ws_bytes)
    torch.cuda.synchronize()
    prob = {n: B.make_problem(B.F16, i, o, r, L, T, workspace=ws, workspace_bytes=ws_bytes,
                              max_seg_len=max(seg_lens), workspace_ready=1) for n, (i, o) in shapes.items()}
    stream = torch.cuda.Stream(device=dev)
    sh = stream.cuda_stream

    def inputs(n):
        # activations a projection reads: x for q/k/v/gate/up, the q output for o (stand-in for
        # the attention output), the up output for down
        return y["q"] if n == "o" else y["up"] if n == "down" else x

    def backbone(l, names):
        for n in names:
            torch.matmul(inputs(n), W[n][l], out=y[n])

    def single(l, n):
        B.sgmv_add_lora(prob[n], y[n], inputs(n), A_ptrs[n], B_ptrs[n], seg_starts, n_req, l, 1.0, sh)

    def multi(l, names):
        B.sgmv_add_lora_multi(prob[names[0]], [y[n] for n in names], [inputs(n) for n in names],
                              [A_ptrs[n] for n in names], [B_ptrs[n] for n in names], seg_starts, n_req, l,
                              1.0, sh)

    def step_backbone(i):
        l = i % L
        backbone(l, ("q", "k", "v")); backbone(l, ("o",)); backbone(l, ("gate", "up")); backbone(l, ("down",))

    def step_single(i):
        l = i % L
        backbone(l, ("q", "k", "v"))
        for n in ("q", "k", "v"):
            single(l, n)
        backbone(l, ("o",)); single(l, "o")
        backbone(l, ("gate", "up")); single(l, "gate"); single(l, "up")
        backbone(l, ("down",)); single(l, "down")

    def step_multi(i):
        l = i % L
        backbone(l, ("q", "k", "v")); multi(l, ("q", "k", "v"))
        backbone(l, ("o",)); single(l, "o")
        backbone(l, ("gate", "up")); multi(l, ("gate", "up"))
        backbone(l, ("down",)); single(l, "down")

    def lora_only_multi(i):
        l = i % L
        multi(l, ("q", "k", "v")); single(l, "o"); multi(l, ("gate", "up")); single(l, "down")

    def timeit(fn):
        K = args.steps
        with torch.cuda.stream(stream):
            for i in range(2 * L):
                fn(i)
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for i in range(K):
                    fn(i)
            g.replay()
            stream.synchronize()
            ts = []
            for _ in range(args.blocks):
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                g.replay()
                e1.record(stream)
                e1.synchronize()
                ts.append(e0.elapsed_time(e1) / K * 1e3)
        return float(np.median(ts))

    res = {"backbone_us": timeit(step_backbone), "lora_single_us": timeit(step_single),
           "lora_multi_us": timeit(step_multi), "lora_only_multi_us": timeit(lora_only_multi)}
    assert B.sgmv_workspace_check(ws, sh) == 0
    weights = sum(i * o for i, o in shapes.values()) * 2
    lora = sum((i * r + r * o) for i, o in shapes.values()) * 2 * n_req
    out = {"benchmark": "decoder-layer dense projections + LoRA add-ons",
           "model": args.model, "h": h, "ffn": ffn, "batch": args.batch, "seq": args.seq, "mix": args.mix,
           "adapters": n_req, "tokens": T, "rank": r,
           "layers_cycled": L,
           "steps": args.steps, "dtype": "f16", "data": "synthetic", "n_gpus": 1,
           "backbone_weight_bytes_per_step": weights, "adapter_weight_bytes_per_step": lora,
           **res,
           "lora_overhead_single_us": res["lora_single_us"] - res["backbone_us"],
           "lora_overhead_multi_us": res["lora_multi_us"] - res["backbone_us"],
           "lora_overhead_multi_frac": res["lora_multi_us"] / res["backbone_us"] - 1.0}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
