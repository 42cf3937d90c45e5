"""The entry point that allocates nothing: sgmv_add_lora_static keeps its intermediate results
in a fixed array inside the library.  Checked through the C ABI against sgmv_add_lora (same
kernels: the bits must agree) and against the CPU oracle, on calls in a row that share the
array, the later ones with smaller inputs."""
import numpy as np
import pytest
import torch

import oracle
import sgmv_workloads as wl
from helpers import decode64, tolerance

pytestmark = pytest.mark.gpu


def _static(d, layer=0, k=0, stream=None):
    from paper_2310_18547_amd import binding as B
    return B.sgmv_add_lora_static(d.problem, d.y[k], d.x[k], d.A_ptrs, d.B_ptrs, d.seg_starts,
                                  d.w.n_segs, layer, d.w.scale, stream)


def _check(w, layer=0, **kw):
    from paper_2310_18547_amd.device import DeviceWorkload
    d = DeviceWorkload(w, "cuda:0", n_sets=2, **kw)
    d.add_lora(layer, 0)                       # the existing entry point, caller's workspace
    _static(d, layer, 1)                       # the same call on the library's array
    want, got = d.y_bits(0), d.y_bits(1)
    ref = oracle.run_workload(w, layer_idx=layer, n_threads=8)
    g, r = decode64(got, w.dtype), decode64(ref, w.dtype)
    assert np.all(np.abs(g - r) <= tolerance(r)), w.name
    assert np.array_equal(got, want), w.name   # same kernels, same summation order
    return d


def test_two_calls_in_a_row_the_second_smaller():
    # single-launch vector kernel, 64 then 7 single-row segments
    _check(wl.decode_distinct(batch=64, h_in=4096, r=16, dtype="f16", num_layers=2, seed=3), 1)
    _check(wl.decode_distinct(batch=7, h_in=4096, r=16, dtype="f16", num_layers=2, seed=4), 1)
    # the rank and the batch change: every region of the array is laid out afresh
    _check(wl.decode_distinct(batch=16, h_in=2048, h_out=1024, r=64, dtype="bf16", num_layers=1, seed=5))
    _check(wl.decode_distinct(batch=3, h_in=512, h_out=768, r=8, dtype="bf16", num_layers=1, seed=6))


def test_every_kernel_family_on_the_static_array():
    from paper_2310_18547_amd import binding as B
    # segments of a few rows: the hand-off kernel per row of the batch, then a smaller mix
    _check(wl.popularity("skewed", batch=64, h_in=4096, r=16, dtype="f16", num_layers=1, seed=5))
    _check(wl.custom([3, 1, 0, 5, 2], 1024, 1536, 32, "bf16", seed=7))
    # the single-launch MFMA tile kernel on the same kind of batch, then on a larger one
    _check(wl.popularity("skewed", batch=64, h_in=4096, r=16, dtype="f16", num_layers=1, seed=5), path=B.PATH_FUSED)
    _check(wl.custom([70, 33, 1, 150, 96, 64, 12, 100], 1024, 768, 16, "bf16", seed=14))
    # launch-per-step MFMA kernels (long segments), then shorter ones
    _check(wl.custom([300, 170, 33], 1024, 768, 16, "bf16", seed=8), path=B.PATH_MATRIX)
    _check(wl.custom([40, 9], 512, 264, 64, "f16", seed=9), path=B.PATH_MATRIX)
    # no length hint: per row in a small batch, the launch-per-step vector kernels in a larger one
    _check(wl.custom([2, 5, 1, 1], 1000, 520, 16, "f16", seed=10), max_seg_len_hint=False)
    _check(wl.custom([2, 5, 1, 1] * 100, 1000, 520, 16, "f16", seed=15), max_seg_len_hint=False)
    _check(wl.custom([1, 1], 256, 256, 8, "f16", seed=11), path=B.PATH_VECTOR)


def test_repeated_calls_and_graph_replay():
    from paper_2310_18547_amd.device import DeviceWorkload
    w = wl.decode_distinct(batch=32, h_in=4096, r=16, dtype="f16", num_layers=4, seed=12)
    d = DeviceWorkload(w, "cuda:0", n_sets=1)
    stream = torch.cuda.Stream(device="cuda:0")
    with torch.cuda.stream(stream):
        _static(d, 0, 0, stream.cuda_stream)   # the array is known by now; this call is eager
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for layer in range(4):
                _static(d, layer, 0, stream.cuda_stream)
        for rep in range(3):
            d.reset_y()
            torch.cuda.synchronize()
            g.replay()
            stream.synchronize()
            # four add-ons on top of each other: compare with the oracle applied four times
            y = w.y0.copy()
            keep = w.y0
            for layer in range(4):
                w.y0 = y
                y = oracle.run_workload(w, layer_idx=layer, n_threads=8)
            w.y0 = keep
            got, ref = decode64(d.y_bits(), "f16"), decode64(y, "f16")
            assert np.all(np.abs(got - ref) <= 4 * tolerance(ref)), f"replay {rep}"


def test_size_limit_and_argument_errors():
    from paper_2310_18547_amd import binding as B
    from paper_2310_18547_amd.device import DeviceWorkload
    w = wl.decode_distinct(batch=4, h_in=256, r=16, dtype="f16", num_layers=1, seed=13)
    d = DeviceWorkload(w, "cuda:0")
    before = d.y_bits().copy()
    p = B.make_problem(B.F16, 256, 256, 64, 1, 4096, max_seg_len=1)      # 4096 tokens at rank 64
    assert B.sgmv_workspace_bytes(4096, 64) > B.STATIC_MAX_WORKSPACE_BYTES
    assert B.sgmv_add_lora_static(p, d.y[0], d.x[0], d.A_ptrs, d.B_ptrs, d.seg_starts, 4, 0, 1.0,
                                  check=False) == 5                      # SGMV_ERR_WORKSPACE
    assert B.sgmv_add_lora_static(d.problem, None, d.x[0], d.A_ptrs, d.B_ptrs, d.seg_starts, 4, 0,
                                  1.0, check=False) == 1                 # SGMV_ERR_NULL
    assert B.sgmv_add_lora_static(d.problem, d.y[0], d.x[0], d.A_ptrs, d.B_ptrs, d.seg_starts, 4, 7,
                                  1.0, check=False) == 6                 # SGMV_ERR_RANGE
    assert np.array_equal(d.y_bits(), before)
    # no workspace in the descriptor at all
    q = B.make_problem(B.F16, 256, 256, 16, 1, 4, max_seg_len=1)
    B.sgmv_add_lora_static(q, d.y[0], d.x[0], d.A_ptrs, d.B_ptrs, d.seg_starts, 4, 0, 1.0)
    got, ref = decode64(d.y_bits(), "f16"), decode64(oracle.run_workload(w), "f16")
    assert np.all(np.abs(got - ref) <= tolerance(ref))
