#!/usr/bin/env python3
"""Benchmark of the SGMV hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One *step* is one pass of the whole hot path: one ``sgmv_add_lora`` call
(segment lookup, shrink, expand) over one batch of synthetic tokens.  The
default workload is the configuration the headline metric is quoted on: Llama-7B
decode shape, Distinct adapters, h_in = h_out = 4096, r = 16, 64 tokens, fp16,
32 layers behind every adapter pointer.  Consecutive steps cycle over the 32
layers (512 MiB of adapter weights) and over several x / y buffer sets, so that
every step streams its weights from HBM rather than from the on-die caches.

Inputs are resident in HBM before the timed region starts.  The K timed steps
are recorded once into a HIP graph and replayed, so the host's launch cost is
outside the measurement; ``--mode eager`` times plain back-to-back calls
instead.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a
# 64 MiB + 64 MiB copy kernel), from the summaries under profiles/; reported as roofline.traffic
MEASURED_TRAFFIC = {"distinct_b64": 18733837.0}
MFMA_PEAK_TFLOPS = 2500.0   # dense bf16 / fp16, MI355X

# the paper's own latencies for this operator (one A100 80 GB, fp16, r = 16), context only
PAPER_A100_US = {"distinct_b64": [116.0, 75.0], "distinct_b1": [37.0, 42.0]}


def make_workload(name: str, seed: int):
    import sgmv_workloads as wl
    if name == "distinct_b64":
        return wl.decode_distinct(batch=64, h_in=4096, r=16, dtype="f16", num_layers=32, seed=seed)
    if name.startswith("distinct_b"):
        return wl.decode_distinct(batch=int(name[len("distinct_b"):]), h_in=4096, r=16,
                                  dtype="f16", num_layers=32, seed=seed)
    if name in ("uniform", "skewed", "identical", "uniform_paper", "skewed_paper"):
        return wl.popularity(name, batch=64, h_in=4096, r=16, dtype="f16", num_layers=32, seed=seed)
    if name == "tiny":
        return wl.tiny(seed=seed)
    if name.startswith("prefill"):
        # prefill_r16, prefill_r64, prefill_mlp_r16, prefill_mlp_r64
        r = int(name.rsplit("r", 1)[1])
        h_out = 28672 if "mlp" in name else 8192
        return wl.prefill(h_in=8192, h_out=h_out, r=r, dtype="bf16", num_layers=1, seed=seed)
    raise SystemExit(f"unknown workload {name!r}")


def cpu_baseline(w, budget_s: float):
    """The oracle as it stands, timed on the host cores over a bounded number of
    add-on calls of the same workload (layers cycled like the GPU loop)."""
    import oracle
    cores = min(os.cpu_count() or 1, 16)
    A_list = [None if a < 0 else w.A[a] for a in w.seg_adapter]
    B_list = [None if a < 0 else w.B[a] for a in w.seg_adapter]
    y = w.y0.copy()
    oracle.add_lora(w.dtype, y, w.x, A_list, B_list, w.seg_starts, 0, w.scale, False, cores)  # warm
    calls, t0 = 0, time.perf_counter()
    while True:
        oracle.add_lora(w.dtype, y, w.x, A_list, B_list, w.seg_starts, calls % w.num_layers,
                        w.scale, False, cores)
        calls += 1
        el = time.perf_counter() - t0
        if el >= budget_s or calls >= 2000:
            break
    from paper_2310_18547_amd import accounting as acc
    by = acc.algorithmic_bytes("add_lora", w.n_tokens, w.n_distinct, w.h_in, w.h_out, w.r)
    # the metric's unit: algorithmic bytes of the same call per second
    return {"value": by * calls / el / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "us_per_call": el / calls * 1e6, "calls_per_s": calls / el,
            "sample": f"{calls} add_lora calls of the same workload ({w.name}), layers cycled, "
                      f"fp32 accumulation, rows split over {cores} threads"}


def time_comparators(d, w, stream, L, S, steps=200):
    """Loop and Gather-BMM (library GEMMs through PyTorch) on the same device tensors:
    microseconds per add-on, eager launches and, where capture works, a replayed HIP graph."""
    import numpy as np
    import torch
    from paper_2310_18547_amd.comparators import Comparators
    c = Comparators(d)
    res = {"note": "PyTorch ops (rocBLAS / hipBLASLt), same GPU and inputs; 16-bit intermediate"}
    for name, fn in (("loop", c.loop), ("gather_bmm", c.gather_bmm)):
        with torch.cuda.stream(stream):
            for i in range(5):
                fn(i % L, i % S)
            stream.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for i in range(steps):
                fn(i % L, i % S)
            e1.record(stream)
            e1.synchronize()
            res[name + "_eager_us"] = e0.elapsed_time(e1) / steps * 1e3
            try:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for i in range(steps):
                        fn(i % L, i % S)
                g.replay()
                stream.synchronize()
                ts = []
                for _ in range(3):
                    e0.record(stream)
                    g.replay()
                    e1.record(stream)
                    e1.synchronize()
                    ts.append(e0.elapsed_time(e1) / steps * 1e3)
                res[name + "_graph_us"] = float(np.median(ts))
            except Exception as exc:  # capture of library calls is not guaranteed
                res[name + "_graph_us"] = None
                res[name + "_graph_error"] = str(exc)[:120]
                torch.cuda.synchronize()
    d.reset_y()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3200)
    ap.add_argument("--warmup", type=int, default=320)
    ap.add_argument("--workload", default="distinct_b64")
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph")
    ap.add_argument("--sets", type=int, default=8, help="x / y buffer sets to rotate over")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ksplit", type=int, default=0)
    ap.add_argument("--expand-threads", type=int, default=0)
    ap.add_argument("--path", type=int, default=0)
    ap.add_argument("--blocks", type=int, default=5, help="timed repetitions; the median is reported")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 64 MiB read + 64 MiB write elementwise kernel, as the "
                         "known-size reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--projections", type=int, default=1,
                    help="add-ons of the same shape per step through sgmv_add_lora_multi (q/k/v = 3); "
                         "1 = the headline metric, one sgmv_add_lora call per step")
    ap.add_argument("--compare", action="store_true",
                    help="also time the paper's two comparison implementations (Loop and Gather-BMM, "
                         "PyTorch library ops) on the same inputs; reported under 'comparators'")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch measured with rocprofv3 --pmc (reported as "
                         "roofline.traffic)")
    args = ap.parse_args()

    if args.gpus != 1:
        raise SystemExit("bench.py measures the single-GPU SGMV kernels only; run with --gpus 1 "
                         "(this build has no multi-GPU path: segments shard across GPUs by "
                         "routing whole requests, with no collective)")

    import numpy as np
    import torch
    from paper_2310_18547_amd import accounting as acc
    from paper_2310_18547_amd.device import DeviceWorkload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = make_workload(args.workload, args.seed)
    d = DeviceWorkload(w, "cuda:0", n_sets=args.sets, path=args.path, ksplit=args.ksplit,
                       expand_threads=args.expand_threads)
    L, S = w.num_layers, args.sets
    stream = torch.cuda.Stream(device="cuda:0")          # default priority
    sh = stream.cuda_stream
    P = args.projections
    if P > 1:
        # P add-ons with their own adapters and outputs, sharing x and the segment indices
        from paper_2310_18547_amd import binding as B
        others = [DeviceWorkload(make_workload(args.workload, args.seed + 1 + i), "cuda:0",
                                 n_sets=args.sets) for i in range(P - 1)]
        ds = [d] + others

        def step(i):
            k = i % S
            B.sgmv_add_lora_multi(d.problem, [q.y[k] for q in ds], [d.x[k]] * P,
                                  [q.A_ptrs for q in ds], [q.B_ptrs for q in ds], d.seg_starts,
                                  w.n_segs, i % L, w.scale, sh)
    else:
        def step(i):
            d.add_lora(i % L, i % S, stream=sh)

    if args.calibrate_copy:
        src = torch.ones(16 << 20, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.add(src, 1, out=dst)            # reads 64 MiB, writes 64 MiB
        torch.cuda.synchronize()

    K, W = args.steps, args.warmup
    with torch.cuda.stream(stream):
        for i in range(W):
            step(i)
        stream.synchronize()
        graph = None
        if args.mode == "graph":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(K):
                    step(i)
            graph.replay()                                   # untimed first replay
            stream.synchronize()

        times = []
        for _ in range(args.blocks):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            if graph is not None:
                graph.replay()
            else:
                for i in range(K):
                    step(i)
            e1.record(stream)
            e1.synchronize()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
    ms_total = float(np.median(times))
    ms_per_step = ms_total / K
    us = ms_per_step * 1e3

    T, n = w.n_tokens, w.n_distinct
    bytes_step = P * acc.algorithmic_bytes("add_lora", T, n, w.h_in, w.h_out, w.r)
    # which kernels the library launched for this call: asked of the library, not re-derived
    from paper_2310_18547_amd import binding as B
    plan = B.sgmv_plan_add_lora(d.problem, w.n_segs, P)
    kernel = {B.KERNEL_FUSED: "add_lora_fused_kernel", B.KERNEL_TILE: "add_lora_tile_kernel",
              B.KERNEL_MULTI_SIDE: "add_lora_fused_side_kernel",
              B.KERNEL_MULTI_PIPELINED: "add_lora_fused_multi_kernel",
              B.KERNEL_VECTOR: "shrink_vector_kernel + expand_vector_kernel",
              B.KERNEL_MATRIX: "shrink_stream_kernel + finalize_v_kernel + expand_matrix_kernel",
              }[plan.kernel]
    launches = plan.launches
    traffic = args.traffic_bytes
    if traffic is None and P == 1 and args.path == 0 and args.ksplit == 0:
        traffic = MEASURED_TRAFFIC.get(args.workload)
    gbs = bytes_step / (ms_per_step * 1e-3) / 1e9

    out = {
        "metric": "SGMV shrink+expand us/layer & HBM GB/s, h=4096 r=16 bs=64 Distinct",
        "value": gbs,
        "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": ms_per_step,
        "us_per_layer": us,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if w.dtype == "f16" else "bf16",
        "accumulate": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "h_in": w.h_in, "h_out": w.h_out, "r": w.r,
                   "tokens": T, "segments": w.n_segs, "distinct_adapters": n,
                   "layers_cycled": L, "xy_sets": S, "mode": args.mode,
                   "steps_per_s": 1e3 / ms_per_step,
                   "projections_per_step": P,
                   "algorithmic_bytes_per_step": bytes_step,
                   "flops_per_step": P * acc.flops("add_lora", T, w.h_in, w.h_out, w.r)},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": kernel, "launches_per_step": launches,
                     "slices_per_segment": plan.slices, "workgroups": plan.workgroups,
                     "algorithmic_bytes_per_step": bytes_step,
                     "avg_step_us": us},
        "paper_a100_us": PAPER_A100_US.get(args.workload),
        "block_ms": times,
    }
    if plan.kernel in (B.KERNEL_MATRIX, B.KERNEL_TILE):
        # the contraction runs on the matrix cores; at r FLOP per byte of x and r/2 per byte of
        # y it sits far left of the MFMA ridge (~312 FLOP/B), so HBM stays the binding roofline
        tf = out["config"]["flops_per_step"] / (ms_per_step * 1e-3) / 1e12
        out["roofline"]["mfma"] = {"achieved": tf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": tf / MFMA_PEAK_TFLOPS,
                                   "flop_per_byte": out["config"]["flops_per_step"] / bytes_step}
    if args.compare:
        out["comparators"] = time_comparators(d, w, stream, L, S)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
