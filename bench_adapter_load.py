#!/usr/bin/env python3
"""On-demand adapter loading next to running SGMV calls.

    python bench_adapter_load.py [--model 7b|13b] [--rank 16] [--batch 64]

The paper loads a LoRA model's weights from host memory when a request for it arrives, with
an asynchronous host-to-device copy that overlaps the running batch (section "On-demand
loading of LoRA models": about 50 us per layer and 2 ms per model over PCIe Gen4 x16).  Here:

* the time to copy ONE adapter (A and B of the seven projections of every layer, one
  contiguous pinned host buffer per projection) to the GPU, per layer and per model;
* the latency of ``sgmv_add_lora`` at the metric shape while such copies run on a second
  stream of default priority, against its latency alone.

The new adapter becomes usable by writing its device pointers into the pointer arrays
(``A_ptrs`` / ``B_ptrs``) before the next call; no kernel or library state is involved.
Prints ONE JSON line.  Synthetic weights; one GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MODELS = {"7b": (4096, 11008, 32), "13b": (5120, 13824, 40)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", choices=sorted(MODELS), default="7b")
    ap.add_argument("--rank", type=int, default=16)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--steps", type=int, default=2000)
    args = ap.parse_args()

    import numpy as np
    import torch
    import sgmv_workloads as wl
    from paper_2310_18547_amd.device import DeviceWorkload

    assert torch.cuda.is_available(), "bench_adapter_load.py needs a GPU"
    dev = torch.device("cuda:0")
    h, ffn, n_layers = MODELS[args.model]
    r = args.rank
    shapes = [(h, h)] * 4 + [(h, ffn)] * 2 + [(ffn, h)]
    # one adapter on the host: per projection [layers][h_in*r + r*h_out] 16-bit, pinned
    host = [torch.empty(n_layers, (i + o) * r, dtype=torch.int16).pin_memory() for i, o in shapes]
    for t in host:
        t.fill_(1)
    devbuf = [torch.empty_like(t, device=dev) for t in host]
    bytes_model = sum(t.numel() * 2 for t in host)
    copy_stream = torch.cuda.Stream(device=dev)

    def load_adapter():
        with torch.cuda.stream(copy_stream):
            for src, dst in zip(host, devbuf):
                dst.copy_(src, non_blocking=True)

    # ---- copy alone
    for _ in range(3):
        load_adapter()
    copy_stream.synchronize()
    reps = 20
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record(copy_stream)
    for _ in range(reps):
        load_adapter()
    e1.record(copy_stream)
    e1.synchronize()
    model_us = e0.elapsed_time(e1) / reps * 1e3

    # ---- add_lora alone, then with copies running on the other stream
    w = wl.decode_distinct(batch=args.batch, h_in=h, r=r, dtype="f16", num_layers=8, seed=0)
    d = DeviceWorkload(w, "cuda:0", n_sets=8)
    stream = torch.cuda.Stream(device=dev)
    K = args.steps

    def timed(with_copies):
        with torch.cuda.stream(stream):
            for i in range(16):
                d.add_lora(i % 8, i % 8, stream=stream.cuda_stream)
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for i in range(K):
                    d.add_lora(i % 8, i % 8, stream=stream.cuda_stream)
            g.replay()
            stream.synchronize()
            ts = []
            for _ in range(3):
                a = torch.cuda.Event(enable_timing=True)
                b = torch.cuda.Event(enable_timing=True)
                if with_copies:                      # enough copies to cover the whole replay
                    for _ in range(max(2, int(K * 8 / model_us) + 2)):
                        load_adapter()
                a.record(stream)
                g.replay()
                b.record(stream)
                b.synchronize()
                copy_stream.synchronize()
                ts.append(a.elapsed_time(b) / K * 1e3)
        return float(np.median(ts))

    alone = timed(False)
    overlapped = timed(True)
    assert d.check() == 0
    out = {"benchmark": "on-demand adapter load (pinned host -> HBM) and its overlap with sgmv_add_lora",
           "model": args.model, "rank": r, "layers": n_layers, "adapter_bytes": bytes_model,
           "load_model_us": model_us, "load_layer_us": model_us / n_layers,
           "load_GBps": bytes_model / model_us / 1e3,
           "add_lora_alone_us": alone, "add_lora_during_loads_us": overlapped,
           "batch": args.batch, "data": "synthetic", "n_gpus": 1,
           "paper_a100_pcie4": {"load_layer_us": 50, "load_model_us": 2000}}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
