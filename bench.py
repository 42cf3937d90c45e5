#!/usr/bin/env python3
"""Benchmark of the SGMV hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--op OP]

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
instead.  After the timed region the workspace's health check must pass and one
fresh call is compared with the CPU oracle element by element.  Prints ONE JSON
line.

Other modes (each prints JSON lines):
    --op shrink|expand|all   the stand-alone entry points (``all``: three lines)
    --table                  every row of the measurement table, one process per workload
    --probe                  launch cost and attainable streaming bandwidth (sgmv_probe)
    --timeline               in-kernel timeline of one call (needs the trace build:
                             python -m paper_2310_18547_amd.build --trace)
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 / fp16, MI355X

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (scaled by the copy
# kernel of sgmv_probe), keyed by what was profiled: (workload, op, kernel, slices).  A run
# whose plan differs from the profiled one reports null.  Source: the summaries in profiles/.
PROFILED_TRAFFIC = {
    ("distinct_b64", "add_lora", "add_lora_fused_kernel", 4):
        (18.620e6, "profiles/add_lora_fused_distinct_b64_h4096_r16.md"),
    ("distinct_b64_r8", "add_lora", "add_lora_whole_kernel", 4):
        (10.086e6, "profiles/add_lora_whole_distinct_b64_h4096_r8.md"),
    ("distinct_b256", "add_lora", "add_lora_whole_kernel", 1):
        (73.658e6, "profiles/add_lora_whole_distinct_b256_h4096_r16.md"),
}

# the paper's own latencies for this operator (one A100 80 GB, fp16, r = 16), context only
PAPER_A100_US = {"distinct_b64": [116.0, 75.0], "distinct_b1": [37.0, 42.0]}

KERNEL_NAMES = None  # filled after the binding is imported


def expand_kernel_name(w) -> str:
    """The MFMA expand kernel the library runs for this workload (rank 64 and binary16 with segments of at least a 64-row block: row-wise)."""
    return "expand_rowwise_kernel" if (w.r > 32 or w.dtype == "f16") and w.max_seg_len >= 64 else "expand_matrix_kernel"


def make_workload(name: str, seed: int, layers: int = 0):
    """Named workloads.  Generic decode shapes: distinct_b{B}[_h{H}][_o{H_OUT}][_r{R}][_{dtype}]."""
    import sgmv_workloads as wl
    kinds = ("uniform_paper", "skewed_paper", "uniform", "skewed", "identical")
    kind = next((k for k in kinds if name == k or name.startswith(k + "_")), None)
    if kind is not None:
        # adapter-popularity mixes: <kind>[_b<batch>][_r<rank>], defaults batch 64, rank 16
        batch, r = 64, 16
        for part in name[len(kind):].split("_")[1:]:
            if part[0] == "b":
                batch = int(part[1:])
            elif part[0] == "r":
                r = int(part[1:])
            else:
                raise SystemExit(f"unknown workload {name!r}")
        return wl.popularity(kind, batch=batch, h_in=4096, r=r, dtype="f16",
                             num_layers=layers or (32 if r <= 16 else 8), seed=seed)
    if name == "tiny":
        return wl.tiny(seed=seed)
    if name.startswith("prefill"):
        # prefill_r16, prefill_r64, prefill_mlp_r16, prefill_mlp_r64; bf16 unless the name ends in _f16
        dtype = "f16" if name.endswith("_f16") else "bf16"
        r = int(name[:-4].rsplit("r", 1)[1] if name.endswith("_f16") else name.rsplit("r", 1)[1])
        h_out = 28672 if "mlp" in name else 8192
        return wl.prefill(h_in=8192, h_out=h_out, r=r, dtype=dtype, num_layers=layers or 1, seed=seed)
    if name.startswith("distinct_b"):
        batch, h, h_out, r, dtype = None, 4096, None, 16, "f16"
        for part in name.split("_")[1:]:
            if part in ("f16", "bf16"):
                dtype = part
            elif part[0] == "b":
                batch = int(part[1:])
            elif part[0] == "h":
                h = int(part[1:])
            elif part[0] == "o":
                h_out = int(part[1:])
            elif part[0] == "r":
                r = int(part[1:])
            else:
                raise SystemExit(f"unknown workload {name!r}")
        if not layers:
            # as many layers as keep the cycled weights beyond the 256 MB Infinity Cache
            per_layer = batch * (h * r + r * (h_out or h)) * 2
            layers = max(1, min(32, -(-(600 << 20) // per_layer)))
        return wl.decode_distinct(batch=batch, h_in=h, h_out=h_out, r=r, dtype=dtype,
                                  num_layers=layers, seed=seed)
    raise SystemExit(f"unknown workload {name!r}")


# rows of the measurement table: (workload name, ops)
TABLE_ROWS = (
    [("tiny", "all")]
    + [(f"distinct_b{b}", "all") for b in (1, 8, 16, 32, 64)]
    + [(k, "all") for k in ("uniform", "skewed", "identical", "uniform_paper", "skewed_paper")]
    + [(f"distinct_b{b}_h{h}_r{r}", "all") for h in (4096, 5120) for r in (8, 32, 64) for b in (16, 64)]
    + [(f"distinct_b{b}", "all") for b in (128, 256, 512, 1024)]
    + [("distinct_b64_bf16", "all"), ("distinct_b64_h5120_bf16", "all")]
    + [(f"distinct_b64_h5120_o13824_r{r}", "all") for r in (16, 64)]       # MLP-shaped expand
    + [(f"distinct_b64_h13824_o5120_r{r}", "all") for r in (16, 64)]       # MLP-shaped shrink
    + [(f"distinct_b64_h4096_o11008_r{r}", "add_lora") for r in (16, 64)]  # Llama-7B gate / up
    + [(f"distinct_b64_h11008_o4096_r{r}", "add_lora") for r in (16, 64)]  # Llama-7B down
    + [(f"prefill_{m}r{r}", "all") for m in ("", "mlp_") for r in (16, 64)]
)


def cpu_baseline(w, budget_s: float, op: str = "add_lora"):
    """The oracle as it stands, timed on the host cores over a bounded number of calls of the
    same workload (layers cycled like the GPU loop): all cores, then one thread."""
    import numpy as np
    import oracle
    from paper_2310_18547_amd import accounting as acc
    cores = min(os.cpu_count() or 1, 16)
    A_list = [None if a < 0 else w.A[a] for a in w.seg_adapter]
    B_list = [None if a < 0 else w.B[a] for a in w.seg_adapter]
    y = w.y0.copy()
    v = np.zeros((w.n_tokens, w.r), np.float32)

    def call(layer, threads):
        if op == "shrink":
            oracle.shrink(w.dtype, v, w.x, A_list, w.seg_starts, layer, False, threads)
        elif op == "expand":
            oracle.expand(w.dtype, y, v, B_list, w.seg_starts, layer, w.scale, False, threads)
        else:
            oracle.add_lora(w.dtype, y, w.x, A_list, B_list, w.seg_starts, layer, w.scale, False, threads)

    def timed(threads, budget, most):
        call(0, threads)  # warm
        calls, t0 = 0, time.perf_counter()
        while True:
            call(calls % w.num_layers, threads)
            calls += 1
            el = time.perf_counter() - t0
            if el >= budget or calls >= most:
                return calls, el

    calls, el = timed(cores, budget_s * 0.7, 2000)
    calls1, el1 = timed(1, budget_s * 0.3, 200)
    by = acc.algorithmic_bytes(op, w.n_tokens, w.n_distinct, w.h_in, w.h_out, w.r)
    # the metric's unit: algorithmic bytes of the same call per second
    return {"value": by * calls / el / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
            "us_per_call": el / calls * 1e6, "calls_per_s": calls / el,
            "single_thread": {"value": by * calls1 / el1 / 1e9, "unit": "GB/s", "cores": 1,
                              "us_per_call": el1 / calls1 * 1e6, "calls": calls1},
            "sample": f"{calls} {op} calls of the same workload ({w.name}), layers cycled, fp32 "
                      f"accumulation, rows split over {cores} threads; then {calls1} calls on one thread"}


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


def timed_graph(stream, step, K, W, blocks, mode="graph"):
    """Median over `blocks` of the milliseconds K steps take on `stream` (HIP events recorded on
    that stream), after W warm-up steps; graph mode replays one captured graph of K steps."""
    import numpy as np
    import torch
    with torch.cuda.stream(stream):
        for i in range(W):
            step(i)
        stream.synchronize()
        graph = None
        if mode == "graph":
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                for i in range(K):
                    step(i)
            graph.replay()                                   # untimed first replay
            stream.synchronize()
        times = []
        for _ in range(blocks):
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
    return float(np.median(times)), times


class Probe:
    """sgmv_probe on a buffer large enough that consecutive launches never read what the
    Infinity Cache still holds."""

    def __init__(self, span_bytes=2 << 30):
        import torch
        self.span = span_bytes
        self.buf = torch.empty(span_bytes, dtype=torch.uint8, device="cuda:0")
        self.buf.fill_(1)
        self.dst = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")
        self.stream = torch.cuda.Stream(device="cuda:0")

    def time_us(self, kind, nbytes, K=400, blocks=3):
        from paper_2310_18547_amd import binding as B
        nbytes = max(16, nbytes // 16 * 16)
        slots = max(1, self.span // max(nbytes, 1))
        base = self.buf.data_ptr()
        dst = self.dst.data_ptr() if kind == B.PROBE_COPY else None
        sh = self.stream.cuda_stream

        def step(i):
            B.sgmv_probe(kind, base + (i % slots) * nbytes, dst, nbytes, sh)

        ms, _ = timed_graph(self.stream, step, K, 20, blocks)
        return ms / K * 1e3


def run_probe(args):
    import torch
    from paper_2310_18547_amd import binding as B
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    p = Probe()
    out = {"benchmark": "sgmv_probe: launch cost and attainable streaming bandwidth, HIP-graph replay, "
                        "buffers rotated over 2 GiB", "n_gpus": 1,
           "empty_us": p.time_us(B.PROBE_EMPTY, 0), "read": [], "copy": []}
    for mib in (1, 4, 9, 16, 18, 32, 64, 256):
        us = p.time_us(B.PROBE_READ, mib << 20)
        out["read"].append({"MiB": mib, "us": us, "GB/s": (mib << 20) / us / 1e3})
    for mib in (16, 64):
        us = p.time_us(B.PROBE_COPY, mib << 20, K=200)
        out["copy"].append({"MiB_read_and_written": mib, "us": us, "GB/s": 2 * (mib << 20) / us / 1e3})
    # one hop of the single-launch kernels' hand-off: a word there and back between two workgroups
    words = torch.zeros(64, dtype=torch.int64, device="cuda:0")
    res = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    out["handoff_round_trip_ns"] = {}
    for partner, where in ((8, "same XCD"), (1, "next XCD"), (4, "XCD four on")):
        trips = []
        for rep in range(5):
            res.zero_()
            B.sgmv_probe(B.PROBE_HANDOFF, words, res, partner)
            torch.cuda.synchronize()
            ticks, gave_up = (int(v) for v in res.cpu())
            assert gave_up == 0
            trips.append(ticks * 10.0 / 200)
        out["handoff_round_trip_ns"][where] = sorted(trips)[len(trips) // 2]
    print(json.dumps(out), flush=True)


def run_timeline(args):
    """One traced call: when the workgroups of the kernel pass the marked points.  Covers the
    single-launch add-on kernels (--op add_lora) and, for long segments, the MFMA shrink
    (--op shrink) and expand (--op expand) kernels of the launch-per-step path."""
    import numpy as np
    import torch
    from paper_2310_18547_amd import binding as B
    from paper_2310_18547_amd.device import DeviceWorkload
    assert "trace" in os.path.basename(B.library_path()), "the timeline needs the trace build"
    w = make_workload(args.workload, args.seed, args.layers)
    d = DeviceWorkload(w, "cuda:0", n_sets=args.sets, path=args.path, ksplit=args.ksplit)
    op = "add_lora" if args.op == "all" else args.op
    if op == "add_lora":
        plan = B.sgmv_plan_add_lora(d.problem, w.n_segs, 1)
        assert plan.launches == 1, "the add_lora timeline covers the single-launch kernels (try --op shrink / expand)"
        n_wg, kernel, slices = plan.workgroups, KERNEL_NAMES[plan.kernel], plan.slices
        call = lambda layer, k: d.add_lora(layer, k)
    else:
        assert w.max_seg_len >= 4, "the shrink / expand timelines cover the MFMA kernels (long segments)"
        n_wg, slices = 1 << 16, None          # an upper bound; workgroups that record nothing are left out
        v = torch.zeros(w.n_tokens, w.r, dtype=torch.float32, device="cuda:0")
        if op == "shrink":
            kernel, call = "shrink_stream_kernel", lambda layer, k: d.shrink(v, layer, k)
        else:
            kernel, call = expand_kernel_name(w), lambda layer, k: d.expand(v, layer, k)
    trace = torch.zeros(n_wg * 10, dtype=torch.int64, device="cuda:0")
    for i in range(64):                       # warm, untraced
        call(i % w.num_layers, i % args.sets)
    torch.cuda.synchronize()
    header = d.workspace[:4352].view(torch.int64)  # generation copies (4 KiB), error word, trace word
    rows = []
    for rep in range(args.blocks):
        trace.zero_()
        header[513] = trace.data_ptr()        # eight bytes behind the error word: trace on
        torch.cuda.synchronize()
        call((7 + rep) % w.num_layers, rep % args.sets)
        torch.cuda.synchronize()
        header[513] = 0
        rows.append(trace.cpu().numpy().reshape(n_wg, 10).astype(np.float64) * 0.01)  # 100 MHz -> us
    assert d.check() == 0
    names = {0: "workgroup started", 8: "segment bounds and pointers known",
             9: "first load about to issue" if kernel == "add_lora_tile_kernel" else "generation tag known (exchange wave)",
             1: "all loads issued",
             2: "x staged in LDS (first data)", 3: "shrink of the slice done", 4: "partial sums published",
             5: "all slices collected", 6: "y stored", 7: "exchange wave leaves"}
    order = [0, 8, 9, 1, 2, 3, 4, 5, 6, 7] if kernel == "add_lora_tile_kernel" else [0, 8, 1, 9, 2, 3, 4, 5, 6, 7]
    if kernel == "add_lora_whole_kernel":      # no hand-off: the workgroup has v once its own waves are summed
        order = [0, 8, 1, 2, 3, 5, 6]
        names[3], names[5] = "shrink done (all of A_i consumed)", "v summed over the waves"
    if op != "add_lora":
        order = [0, 8, 1, 2, 6]
        names[1] = "first tiles and weight loads issued"
        names[2] = "weight slice transposed into LDS"
        names[6] = "last tile done (results stored)"
    points = []
    live_counts = []
    for p_ in order:
        per_rep = []
        for t in rows:
            live = t[:, 6] > 0
            live_counts.append(int(live.sum()))
            t0 = t[live, 0].min()
            per_rep.append(np.percentile(t[live, p_] - t0, [0, 50, 90, 100]))
        q = np.median(np.asarray(per_rep), axis=0)
        points.append({"point": names[p_], "min_us": q[0], "median_us": q[1], "p90_us": q[2], "max_us": q[3]})
    out = {"benchmark": "in-kernel timeline (trace build), microseconds after the first workgroup started",
           "workload": w.name, "kernel": kernel, "workgroups": live_counts[0] if op != "add_lora" else n_wg,
           "slices_per_segment": slices, "traced_calls": len(rows), "points": points}
    print(json.dumps(out), flush=True)


def validate(d, w, op, sh):
    """One fresh call on reset buffers against the CPU oracle, element by element."""
    import numpy as np
    import oracle
    import torch
    tol = lambda ref: 2e-3 + 2e-2 * np.abs(ref)
    dec = lambda bits: (bits.view(np.float16).astype(np.float64) if w.dtype == "f16" else
                        (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64))
    layer = w.num_layers - 1
    d.reset_y(0)
    torch.cuda.synchronize()          # the reset ran on torch's stream, the call below runs on `sh`
    if op == "shrink":
        v = torch.zeros(w.n_tokens, w.r, dtype=torch.float32, device="cuda:0")
        d.shrink(v, layer, 0, stream=sh)
        torch.cuda.synchronize()
        got = v.cpu().numpy().astype(np.float64)
        ref = oracle.run_workload(w, op="shrink", layer_idx=layer, n_threads=16).astype(np.float64)
    elif op == "expand":
        vin = np.random.Generator(np.random.PCG64(5)).standard_normal((w.n_tokens, w.r)).astype(np.float32)
        d.expand(torch.from_numpy(vin).to("cuda:0"), layer, 0, stream=sh)
        got = dec(d.y_bits(0))
        ref = dec(oracle.run_workload(w, op="expand", layer_idx=layer, v=vin, n_threads=16))
    else:
        d.add_lora(layer, 0, stream=sh)
        got = dec(d.y_bits(0))
        ref = dec(oracle.run_workload(w, layer_idx=layer, n_threads=16))
    err = np.abs(got - ref)
    ok = bool(np.all(err <= tol(ref)))
    return {"max_abs_err": float(err.max()) if err.size else 0.0, "within_tolerance": ok,
            "bar": "|gpu - oracle| <= 2e-3 + 2e-2 |oracle|", "elements": int(err.size)}


def bench_one(args, op, d, w, probe):
    import torch
    from paper_2310_18547_amd import accounting as acc
    from paper_2310_18547_amd import binding as B
    L, S = w.num_layers, args.sets
    stream = torch.cuda.Stream(device="cuda:0")          # default priority
    sh = stream.cuda_stream
    P = args.projections if op == "add_lora" else 1
    if P > 1:
        # P add-ons with their own adapters and outputs, sharing x and the segment indices
        from paper_2310_18547_amd.device import DeviceWorkload
        others = [DeviceWorkload(make_workload(args.workload, args.seed + 1 + i, args.layers), "cuda:0",
                                 n_sets=args.sets) for i in range(P - 1)]
        ds = [d] + others

        def step(i):
            k = i % S
            B.sgmv_add_lora_multi(d.problem, [q.y[k] for q in ds], [d.x[k]] * P,
                                  [q.A_ptrs for q in ds], [q.B_ptrs for q in ds], d.seg_starts,
                                  w.n_segs, i % L, w.scale, sh)
    elif op == "shrink":
        v = torch.zeros(w.n_tokens, w.r, dtype=torch.float32, device="cuda:0")

        def step(i):
            d.shrink(v, i % L, i % S, stream=sh)
    elif op == "expand":
        v = torch.randn(w.n_tokens, w.r, dtype=torch.float32, device="cuda:0")

        def step(i):
            d.expand(v, i % L, i % S, stream=sh)
    else:
        def step(i):
            d.add_lora(i % L, i % S, stream=sh)

    K, W = args.steps, args.warmup
    ms_total, times = timed_graph(stream, step, K, W, args.blocks, args.mode)
    ms_per_step = ms_total / K
    us = ms_per_step * 1e3
    health = d.check(sh)
    if health != 0:
        raise SystemExit(f"workspace health check failed after the timed loop: status {health} "
                         f"({B.sgmv_status_string(health)})")

    T, n = w.n_tokens, w.n_distinct
    bytes_step = P * acc.algorithmic_bytes(op, T, n, w.h_in, w.h_out, w.r)
    flops_step = P * acc.flops(op, T, w.h_in, w.h_out, w.r)
    # which kernels the library launched for this call: asked of the library, not re-derived
    if op == "add_lora":
        plan = B.sgmv_plan_add_lora(d.problem, w.n_segs, P)
        kernel, launches, slices, workgroups = KERNEL_NAMES[plan.kernel], plan.launches, plan.slices, plan.workgroups
        if plan.kernel == B.KERNEL_MATRIX:
            kernel = kernel.replace("expand_matrix_kernel", expand_kernel_name(w))
    else:
        if op == "shrink":  # asked of the library
            sp = B.sgmv_plan_shrink(d.problem, w.n_segs)
            long_segments = sp.kernel == B.KERNEL_MATRIX
        else:
            ep = B.sgmv_plan_expand(d.problem, w.n_segs)
            long_segments = ep.kernel == B.KERNEL_MATRIX
        kernel = {("shrink", False): "shrink_vector_kernel + shrink_reduce_kernel",
                  ("shrink", True): "shrink_stream_kernel + shrink_reduce_kernel",
                  ("expand", False): "expand_vector_kernel",
                  ("expand", True): "finalize_v_kernel + " + expand_kernel_name(w)}[(op, long_segments)]
        launches, slices, workgroups = (1 if kernel == "expand_vector_kernel" else 2), None, None
        if op == "expand" and not long_segments and ep.lds_bytes >= 6144:   # the partial sums of three waves are in LDS
            kernel = "expand_split_kernel"
        if op == "shrink" and sp.kernel == B.KERNEL_FUSED:
            kernel, launches, slices, workgroups = "shrink_handoff_kernel", 1, sp.slices, sp.workgroups
        if op == "shrink" and sp.kernel == B.KERNEL_WHOLE:
            kernel, launches, slices, workgroups = "shrink_whole_kernel", 1, sp.slices, sp.workgroups
    traffic = args.traffic_bytes
    traffic_source = "--traffic-bytes" if traffic is not None else None
    if traffic is None and P == 1 and args.path == 0 and args.ksplit == 0:
        hit = PROFILED_TRAFFIC.get((args.workload, op, kernel, slices))
        if hit:
            traffic, traffic_source = hit
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
        "config": {"workload": w.name, "name": args.workload, "op": op, "h_in": w.h_in, "h_out": w.h_out,
                   "r": w.r, "tokens": T, "segments": w.n_segs, "distinct_adapters": n,
                   "layers_cycled": L, "xy_sets": S, "mode": args.mode,
                   "steps_per_s": 1e3 / ms_per_step,
                   "projections_per_step": P,
                   "algorithmic_bytes_per_step": bytes_step,
                   "flops_per_step": flops_step},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gbs / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel, "launches_per_step": launches,
                     "slices_per_segment": slices, "workgroups": workgroups,
                     "algorithmic_bytes_per_step": bytes_step,
                     "avg_step_us": us},
        "paper_a100_us": PAPER_A100_US.get(args.workload) if op == "add_lora" else None,
        "block_ms": times,
    }
    if probe is not None:
        # what a kernel that only reads the same number of bytes reaches on this GPU, one launch
        pus = probe.time_us(B.PROBE_READ, bytes_step)
        out["roofline"]["attainable"] = {
            "what": "sgmv_probe streaming read of the same bytes in one launch, same timing protocol",
            "us": pus, "GB/s": bytes_step / pus / 1e3, "frac_of_peak": bytes_step / pus / 1e3 / HBM_PEAK_GBS,
            "step_over_probe": us / pus, "empty_launch_us": probe.time_us(B.PROBE_EMPTY, 0)}
    if "tile" in kernel or "matrix" in kernel or "stream" in kernel:
        # the contraction runs on the matrix cores; at r FLOP per byte of x and r/2 per byte of
        # y it sits far left of the MFMA ridge (~312 FLOP/B), so HBM stays the binding roofline
        tf = flops_step / (ms_per_step * 1e-3) / 1e12
        out["roofline"]["mfma"] = {"achieved": tf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": tf / MFMA_PEAK_TFLOPS, "flop_per_byte": flops_step / bytes_step}
    if not args.no_validate:
        out["validation"] = validate(d, w, op, sh)
        if not out["validation"]["within_tolerance"]:
            raise SystemExit(f"result outside the parity bar: {out['validation']}")
    if args.compare and op == "add_lora":
        out["comparators"] = time_comparators(d, w, stream, L, S)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds, op)
    return out


def run_table(args):
    """One process per workload (where the allocator puts the weights moves a row by several
    percent), three lines per workload; every line is echoed as it arrives."""
    for name, ops in TABLE_ROWS:
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", name, "--op", ops,
               "--steps", str(args.table_steps), "--warmup", "50", "--blocks", "3", "--no-cpu-baseline"]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            print(json.dumps({"workload": name, "error": (res.stderr or res.stdout)[-400:]}), flush=True)
            continue
        for line in res.stdout.splitlines():
            if line.startswith("{"):
                print(line, flush=True)


def main():
    global KERNEL_NAMES
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3200)
    ap.add_argument("--warmup", type=int, default=320)
    ap.add_argument("--workload", default="distinct_b64")
    ap.add_argument("--op", choices=["add_lora", "shrink", "expand", "all"], default="add_lora")
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph")
    ap.add_argument("--sets", type=int, default=8, help="x / y buffer sets to rotate over")
    ap.add_argument("--layers", type=int, default=0, help="layers behind every adapter pointer (0: per workload)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-validate", action="store_true")
    ap.add_argument("--no-attainable", action="store_true")
    ap.add_argument("--ksplit", type=int, default=0)
    ap.add_argument("--expand-threads", type=int, default=0)
    ap.add_argument("--path", type=int, default=0)
    ap.add_argument("--blocks", type=int, default=5, help="timed repetitions; the median is reported")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 64 MiB copy (sgmv_probe kind 2: reads 64 MiB, writes 64 MiB), the "
                         "known-size reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--projections", type=int, default=1,
                    help="add-ons of the same shape per step through sgmv_add_lora_multi (q/k/v = 3); "
                         "1 = the headline metric, one sgmv_add_lora call per step")
    ap.add_argument("--compare", action="store_true",
                    help="also time the paper's two comparison implementations (Loop and Gather-BMM, "
                         "PyTorch library ops) on the same inputs; reported under 'comparators'")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch measured with rocprofv3 --pmc (reported as roofline.traffic)")
    ap.add_argument("--table", action="store_true")
    ap.add_argument("--table-steps", type=int, default=800)
    ap.add_argument("--probe", action="store_true")
    ap.add_argument("--timeline", action="store_true")
    args = ap.parse_args()

    if args.gpus != 1:
        raise SystemExit("bench.py measures the single-GPU SGMV kernels only; run with --gpus 1 "
                         "(this build has no multi-GPU path: segments shard across GPUs by "
                         "routing whole requests, with no collective)")
    if args.table:
        return run_table(args)
    if args.timeline:
        os.environ.setdefault("SGMV_LIBRARY", "libsgmv_trace.so")

    import torch
    from paper_2310_18547_amd import binding as B
    from paper_2310_18547_amd.device import DeviceWorkload
    KERNEL_NAMES = {B.KERNEL_FUSED: "add_lora_fused_kernel", B.KERNEL_TILE: "add_lora_tile_kernel",
                    B.KERNEL_MULTI_SIDE: "add_lora_fused_side_kernel",
                    B.KERNEL_MULTI_PIPELINED: "add_lora_fused_multi_kernel",
                    B.KERNEL_VECTOR: "shrink_vector_kernel + expand_vector_kernel",
                    B.KERNEL_MATRIX: "shrink_stream_kernel + finalize_v_kernel + expand_matrix_kernel",
                    B.KERNEL_WHOLE: "add_lora_whole_kernel"}
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.probe:
        return run_probe(args)
    if args.timeline:
        return run_timeline(args)

    w = make_workload(args.workload, args.seed, args.layers)
    d = DeviceWorkload(w, "cuda:0", n_sets=args.sets, path=args.path, ksplit=args.ksplit,
                       expand_threads=args.expand_threads, n_proj=args.projections)
    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        B.sgmv_probe(B.PROBE_COPY, src, dst, 64 << 20)
        torch.cuda.synchronize()
    probe = None if args.no_attainable else Probe(1 << 30)
    for op in (["add_lora", "shrink", "expand"] if args.op == "all" else [args.op]):
        print(json.dumps(bench_one(args, op, d, w, probe)), flush=True)


if __name__ == "__main__":
    main()
