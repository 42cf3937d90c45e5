"""Seeded synthetic inputs for SGMV (Punica, arxiv 2310.18547).

This module only *draws and encodes* inputs; it contains none of the operator's
arithmetic.  Both the CPU oracle's tests and the HIP path's tests/bench take
their inputs from here so that the two sides see identical bits.

All 16-bit tensors are handed out as ``numpy.uint16`` bit patterns plus a dtype
tag (``"f16"`` or ``"bf16"``), so neither side depends on the other's number
format code.

Workload shapes follow the paper's evaluation section (microbenchmarks of the
LoRA operator: rank 16, batch 1..64, random LoRA weights, the four adapter
popularity mixes Distinct / Uniform / Skewed / Identical) and the five
configurations this build is measured on.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

DTYPES = ("f16", "bf16")


# --------------------------------------------------------------------------
# encoding of drawn fp32 values into 16-bit storage (input preparation only)
# --------------------------------------------------------------------------
def encode(values_f32: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 samples to the 16-bit storage type, return the bit patterns."""
    v = np.ascontiguousarray(values_f32, dtype=np.float32)
    if dtype == "f16":
        return v.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = v.view(np.uint32)
        rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        return rounded.astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


@dataclass
class Workload:
    """One SGMV problem instance, host side.

    ``A[a]`` is adapter ``a``'s stacked shrink weight ``[num_layers, h_in, r]``
    and ``B[a]`` its expand weight ``[num_layers, r, h_out]`` (row-major bit
    patterns).  ``seg_adapter[i]`` says which adapter segment ``i`` uses; -1
    means "no adapter" (a null pointer in the pointer arrays).
    """

    name: str
    dtype: str
    h_in: int
    h_out: int
    r: int
    num_layers: int
    seg_starts: np.ndarray            # int32 [n_segs + 1]
    seg_adapter: np.ndarray           # int64 [n_segs]
    A: List[np.ndarray]               # per adapter uint16 [L, h_in, r]
    B: List[np.ndarray]               # per adapter uint16 [L, r, h_out]
    x: np.ndarray                     # uint16 [T, h_in]
    y0: np.ndarray                    # uint16 [T, h_out]
    scale: float = 1.0
    seed: int = 0
    notes: dict = field(default_factory=dict)

    @property
    def n_tokens(self) -> int:
        return int(self.seg_starts[-1]) if len(self.seg_starts) else 0

    @property
    def n_segs(self) -> int:
        return len(self.seg_starts) - 1

    @property
    def max_seg_len(self) -> int:
        if self.n_segs <= 0:
            return 0
        return int(np.max(np.diff(self.seg_starts)))

    @property
    def n_distinct(self) -> int:
        """Number of distinct adapters actually touched by non-empty segments."""
        lens = np.diff(self.seg_starts)
        ids = self.seg_adapter[(lens > 0) & (self.seg_adapter >= 0)]
        return int(len(np.unique(ids)))


# --------------------------------------------------------------------------
# building blocks
# --------------------------------------------------------------------------
def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def make_adapters(rng, n_adapters, num_layers, h_in, h_out, r, dtype,
                  want_A=True, want_B=True):
    """A ~ N(0, 1/sqrt(h_in)) std, B ~ N(0, 1/sqrt(r)) std (fan-in scaling)."""
    A, B = [], []
    for _ in range(n_adapters):
        if want_A:
            A.append(encode(_normal(rng, (num_layers, h_in, r), 1.0 / np.sqrt(h_in)), dtype))
        else:
            A.append(np.zeros((num_layers, h_in, r), np.uint16))
        if want_B:
            B.append(encode(_normal(rng, (num_layers, r, h_out), 1.0 / np.sqrt(r)), dtype))
        else:
            B.append(np.zeros((num_layers, r, h_out), np.uint16))
    return A, B


def segments_from_ids(ids: Sequence[int]):
    """Stable-sort adapter ids so equal ids are consecutive; run-length encode.

    Returns (seg_starts int32 [n+1], seg_adapter int64 [n]).  This mirrors how a
    serving batch is ordered before the operator is called: requests to the
    same adapter are placed next to each other and the segment indices are
    built once per model invocation.
    """
    ids = np.sort(np.asarray(ids, dtype=np.int64), kind="stable")
    if ids.size == 0:
        return np.zeros(1, np.int32), np.zeros(0, np.int64)
    change = np.flatnonzero(np.diff(ids)) + 1
    starts = np.concatenate(([0], change, [ids.size])).astype(np.int32)
    return starts, ids[starts[:-1]].astype(np.int64)


def _assemble(name, rng, dtype, h_in, h_out, r, num_layers, seg_starts, seg_adapter,
              n_adapters, scale, seed, notes=None, want_A=True, want_B=True):
    T = int(seg_starts[-1])
    A, B = make_adapters(rng, n_adapters, num_layers, h_in, h_out, r, dtype, want_A, want_B)
    x = encode(_normal(rng, (T, h_in), 1.0), dtype)
    y0 = encode(_normal(rng, (T, h_out), 1.0), dtype)
    return Workload(name=name, dtype=dtype, h_in=h_in, h_out=h_out, r=r,
                    num_layers=num_layers,
                    seg_starts=np.asarray(seg_starts, np.int32),
                    seg_adapter=np.asarray(seg_adapter, np.int64),
                    A=A, B=B, x=x, y0=y0, scale=float(scale), seed=seed,
                    notes=notes or {})


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------
def tiny(seed: int = 0, dtype: str = "f16") -> Workload:
    """Config 1: h=256, r=8, 8 tokens in segments of sizes [1,3,2,2], 4 adapters."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return _assemble("tiny", rng, dtype, 256, 256, 8, 1,
                     [0, 1, 4, 6, 8], [0, 1, 2, 3], 4, 1.0, seed)


def decode_distinct(batch: int = 64, h_in: int = 4096, h_out: Optional[int] = None,
                    r: int = 16, dtype: str = "f16", num_layers: int = 32,
                    seed: int = 0, scale: float = 1.0) -> Workload:
    """Config 2 / 4: every token is its own segment with its own adapter."""
    h_out = h_in if h_out is None else h_out
    rng = np.random.Generator(np.random.PCG64(seed))
    starts = np.arange(batch + 1, dtype=np.int32)
    return _assemble(f"distinct_b{batch}_h{h_in}x{h_out}_r{r}_{dtype}", rng, dtype,
                     h_in, h_out, r, num_layers, starts, np.arange(batch), batch,
                     scale, seed)


def zipf_probabilities(n: int, alpha: float) -> np.ndarray:
    p = 1.0 / np.power(np.arange(1, n + 1, dtype=np.float64), alpha)
    return p / p.sum()


def geometric_counts(batch: int, alpha: float) -> np.ndarray:
    """The paper's *definition* of its skewed mix: the i-th most popular model
    receives alpha times the requests of the (i+1)-th.  Counts are rounded with
    the largest-remainder rule so that they sum to ``batch``."""
    n = batch
    w = np.power(alpha, -np.arange(n, dtype=np.float64))
    ideal = w / w.sum() * batch
    base = np.floor(ideal).astype(np.int64)
    rem = batch - int(base.sum())
    order = np.argsort(-(ideal - base), kind="stable")
    base[order[:rem]] += 1
    return base[base > 0]


def popularity(kind: str, batch: int = 64, pool: int = 64, h_in: int = 4096,
               h_out: Optional[int] = None, r: int = 16, dtype: str = "f16",
               num_layers: int = 32, seed: int = 0, scale: float = 1.0) -> Workload:
    """Config 3: adapter popularity mixes.

    kind:
      "distinct"        one adapter per token
      "uniform"         id per token ~ U{0..pool-1}
      "skewed"          id per token ~ Zipf(1.5) truncated to ``pool`` ids
      "identical"       one segment holding the whole batch
      "uniform_paper"   ceil(sqrt(batch)) equally popular adapters (paper's text)
      "skewed_paper"    geometric counts with ratio 1.5 (paper's definition)
    """
    h_out = h_in if h_out is None else h_out
    rng = np.random.Generator(np.random.PCG64(seed))
    if kind == "distinct":
        ids = np.arange(batch)
    elif kind == "uniform":
        ids = rng.integers(0, pool, size=batch)
    elif kind == "skewed":
        ids = rng.choice(pool, size=batch, p=zipf_probabilities(pool, 1.5))
    elif kind == "identical":
        ids = np.zeros(batch, np.int64)
    elif kind == "uniform_paper":
        m = int(np.ceil(np.sqrt(batch)))
        ids = np.arange(batch) % m
    elif kind == "skewed_paper":
        counts = geometric_counts(batch, 1.5)
        ids = np.repeat(np.arange(len(counts)), counts)
    else:
        raise ValueError(kind)
    starts, seg_ids = segments_from_ids(ids)
    # only materialise the adapters that are used; remap ids to 0..n-1
    uniq, remap = np.unique(seg_ids, return_inverse=True)
    return _assemble(f"{kind}_b{batch}_h{h_in}_r{r}_{dtype}", rng, dtype, h_in, h_out, r,
                     num_layers, starts, remap, len(uniq), scale, seed,
                     notes={"pool_ids": uniq.tolist()})


def prefill(h_in: int = 8192, h_out: int = 8192, r: int = 16, dtype: str = "bf16",
            n_segs: int = 8, min_len: int = 128, max_len: int = 1024,
            num_layers: int = 1, seed: int = 0, scale: float = 1.0) -> Workload:
    """Config 5: a few long segments, lengths ~ U{min_len..max_len}."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = rng.integers(min_len, max_len + 1, size=n_segs)
    starts = np.concatenate(([0], np.cumsum(lens))).astype(np.int32)
    return _assemble(f"prefill_{n_segs}seg_h{h_in}x{h_out}_r{r}_{dtype}", rng, dtype,
                     h_in, h_out, r, num_layers, starts, np.arange(n_segs), n_segs,
                     scale, seed, notes={"seg_lens": lens.tolist()})


def custom(seg_lens: Sequence[int], h_in: int, h_out: int, r: int, dtype: str = "f16",
           num_layers: int = 1, seed: int = 0, scale: float = 1.0,
           seg_adapter: Optional[Sequence[int]] = None, name: str = "custom") -> Workload:
    """Arbitrary segment lengths (zeros allowed) for edge-case tests."""
    rng = np.random.Generator(np.random.PCG64(seed))
    starts = np.concatenate(([0], np.cumsum(np.asarray(seg_lens, np.int64)))).astype(np.int32)
    n = len(seg_lens)
    if seg_adapter is None:
        seg_adapter = np.arange(n)
    seg_adapter = np.asarray(seg_adapter, np.int64)
    n_adapters = int(seg_adapter.max()) + 1 if n and seg_adapter.max() >= 0 else 0
    return _assemble(name, rng, dtype, h_in, h_out, r, num_layers, starts, seg_adapter,
                     n_adapters, scale, seed)


def fingerprint(seg_lens: Sequence[int], h_in: int, h_out: int, r: int, dtype: str = "f16",
                num_layers: int = 1, layer_idx: int = 0) -> Workload:
    """Inputs whose whole computation is exact in 16-bit and fp32 arithmetic.

    Adapter ``a`` at layer ``l`` has A[l, k, j] = 1 only at (k=a mod h_in, j=a mod r)
    and B[l, j, :] = (a + 1) + 32*l on that same j; token ``t`` has x[t, :] = 1 on
    every k, and y0 = 0.  The result y[t, :] then equals ``(a+1) + 32*l`` for
    the adapter/layer the token was really routed to, exactly, so the output
    encodes the routing.
    """
    one = {"f16": 0x3C00, "bf16": 0x3F80}[dtype]
    n = len(seg_lens)
    starts = np.concatenate(([0], np.cumsum(np.asarray(seg_lens, np.int64)))).astype(np.int32)
    T = int(starts[-1])
    A, B = [], []
    for a in range(n):
        Aa = np.zeros((num_layers, h_in, r), np.uint16)
        Ba = np.zeros((num_layers, r, h_out), np.uint16)
        for l in range(num_layers):
            Aa[l, a % h_in, a % r] = one
            val = np.full((h_out,), float(a + 1 + 32 * l), np.float32)
            Ba[l, a % r, :] = encode(val, dtype)
        A.append(Aa)
        B.append(Ba)
    x = np.full((T, h_in), one, np.uint16)
    y0 = np.zeros((T, h_out), np.uint16)
    return Workload(name="fingerprint", dtype=dtype, h_in=h_in, h_out=h_out, r=r,
                    num_layers=num_layers, seg_starts=starts,
                    seg_adapter=np.arange(n, dtype=np.int64), A=A, B=B, x=x, y0=y0,
                    scale=1.0, seed=-1)
