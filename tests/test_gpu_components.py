"""GPU tests of the two rows built around the hot path: on-demand adapter loading next to
running calls, and the seven add-ons of one decoder layer.  Both go through the C ABI and
compare every output with the CPU oracle element by element."""
import numpy as np
import pytest
import torch

import oracle
import sgmv_workloads as wl
from helpers import decode64, tolerance

pytestmark = pytest.mark.gpu


def _assert_parity(got_bits, ref_bits, dtype, what):
    got, ref = decode64(got_bits, dtype), decode64(ref_bits, dtype)
    bad = ~(np.abs(got - ref) <= tolerance(ref))
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance"


# ------------------------------------------------------------ on-demand adapter loading
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_adapter_loaded_on_second_stream_joins_the_batch(dtype):
    from paper_2310_18547_amd.adapter_pool import AdapterPool
    from paper_2310_18547_amd.device import DeviceWorkload
    L, h, r, batch = 3, 2048, 16, 16
    w = wl.decode_distinct(batch=batch, h_in=h, r=r, dtype=dtype, num_layers=L, seed=41)
    d = DeviceWorkload(w, "cuda:0", n_sets=2)
    # two adapters that are not on the device yet: pinned host copies
    rng = np.random.Generator(np.random.PCG64(42))
    newA, newB = wl.make_adapters(rng, 2, L, h, h, r, dtype)
    pool = AdapterPool(2, L, h, h, r, "cuda:0")
    host = [(AdapterPool.pin(a), AdapterPool.pin(b)) for a, b in zip(newA, newB)]
    compute = torch.cuda.Stream(device="cuda:0")     # default priority, both of them
    copy = torch.cuda.Stream(device="cuda:0")

    # a batch is running (set 1 takes the calls whose result is not looked at) ...
    for i in range(50):
        d.add_lora(i % L, 1, stream=compute.cuda_stream)
    # ... while the two adapters arrive on the other stream
    ready = [pool.load_async(s, *host[s], copy) for s in range(2)]
    for i in range(50):
        d.add_lora(i % L, 1, stream=compute.cuda_stream)
    # before the swap the batch still uses the resident adapters
    d.add_lora(2, 0, stream=compute.cuda_stream)
    compute.synchronize()
    _assert_parity(d.y_bits(0), oracle.run_workload(w, layer_idx=2, n_threads=8), dtype, "before the swap")

    # segments 3 and 11 switch to the new adapters; calls enqueued afterwards see them
    d.reset_y(0)
    pool.bind(d.A_ptrs, d.B_ptrs, 3, 0, compute, ready[0])
    pool.bind(d.A_ptrs, d.B_ptrs, 11, 1, compute, ready[1])
    d.add_lora(1, 0, stream=compute.cuda_stream)
    compute.synchronize()
    w.A = list(w.A)
    w.B = list(w.B)
    w.A[3], w.B[3] = newA[0], newB[0]
    w.A[11], w.B[11] = newA[1], newB[1]
    ref = oracle.run_workload(w, layer_idx=1, n_threads=8)
    _assert_parity(d.y_bits(0), ref, dtype, "after the swap")
    # the two swapped rows really changed adapter: they differ from what the old ones give
    assert d.check(compute.cuda_stream) == 0
    copy.synchronize()


# ------------------------------------------------------------ one decoder layer, seven add-ons
@pytest.mark.parametrize("h,ffn,batch,r", [(4096, 11008, 12, 16), (5120, 13824, 5, 8)])
def test_decoder_layer_seven_add_ons(h, ffn, batch, r):
    from paper_2310_18547_amd import binding as B
    from paper_2310_18547_amd.device import DeviceWorkload
    from paper_2310_18547_amd.layer import GROUPS, LoraLayer, projection_shapes
    L, dtype = 2, "f16"
    shapes = projection_shapes(h, ffn)
    ws = {n: wl.decode_distinct(batch=batch, h_in=i, h_out=o, r=r, dtype=dtype, num_layers=L,
                                seed=60 + k) for k, (n, (i, o)) in enumerate(shapes.items())}
    # q, k, v read the same activations, and so do gate and up
    for n in ("k", "v"):
        ws[n].x = ws["q"].x
    ws["up"].x = ws["gate"].x
    ds = {n: DeviceWorkload(w, "cuda:0", init_workspace=False) for n, w in ws.items()}
    layer = LoraLayer(h, ffn, r, L, batch, B.F16, {n: d.A_ptrs for n, d in ds.items()},
                      {n: d.B_ptrs for n, d in ds.items()}, ds["q"].seg_starts, batch, 1)
    stream = torch.cuda.Stream(device="cuda:0")
    for names in GROUPS:
        plan = B.sgmv_plan_add_lora(layer.problem[names[0]], batch, len(names))
        assert plan.launches == 1                      # every group is a single kernel launch
        layer.add_lora_group(names, [ds[n].y[0] for n in names], [ds[names[0]].x[0]] * len(names),
                             1, 1.0, stream.cuda_stream)
    stream.synchronize()
    assert layer.check(stream.cuda_stream) == 0
    for n, w in ws.items():
        _assert_parity(ds[n].y_bits(), oracle.run_workload(w, layer_idx=1, n_threads=8), dtype,
                       f"projection {n} {shapes[n]}")
