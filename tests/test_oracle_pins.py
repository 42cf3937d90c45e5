"""Pins for the CPU oracle (no GPU).

The paper prints no worked numeric example of SGMV, so the oracle is pinned by
what the paper and the mathematics fix:
  * the defining equation of the SGMV section, evaluated by a structurally
    different fp64 brute force on small inputs;
  * the Identical case being one dense product (the LoRA-operator
    microbenchmark paragraph: all implementations reduce to one BMM);
  * the Distinct case being a matrix-vector product per token (last paragraph of
    the SGMV section);
  * grouping being a pure re-ordering (segment definition paragraph):
    permutation and segment-split invariance;
  * exact-integer fingerprints that make every routing decision visible in the
    output bits;
  * linearity of the add-on and the two-launch decomposition v := 0; v += xA;
    y += vB.
"""
import numpy as np
import pytest
import torch

import oracle
import sgmv_workloads as wl
from helpers import brute_force_add_lora, decode64, ulp

DTYPES = ["f16", "bf16"]


# ---------------------------------------------------------------- formats
def test_decode_all_bit_patterns_f16():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.decode(bits, "f16")
    want = bits.view(np.float16).astype(np.float32)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(want)], want.view(np.uint32)[~np.isnan(want)])
    assert np.all(np.isnan(got[np.isnan(want)]))


def test_decode_all_bit_patterns_bf16():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.decode(bits, "bf16")
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    ok = ~np.isnan(want)
    assert np.array_equal(got.view(np.uint32)[ok], want.view(np.uint32)[ok])
    assert np.all(np.isnan(got[~ok]))


def _edge_floats():
    rng = np.random.Generator(np.random.PCG64(11))
    parts = [
        rng.standard_normal(200000).astype(np.float32),
        (rng.standard_normal(100000) * 1e-5).astype(np.float32),          # f16 subnormal range
        (rng.standard_normal(100000) * 3e4).astype(np.float32),           # near f16 overflow
        rng.integers(0, 2**32, 300000, dtype=np.uint64).astype(np.uint32).view(np.float32),
        np.array([0.0, -0.0, np.inf, -np.inf, 65504.0, 65520.0, 65519.99, 2.0**-24, 2.0**-25,
                  2.0**-25 * 1.0000001, 2.0**-14, 2.0**-14 - 2.0**-25, 1.0 + 2.0**-11,
                  1.0 + 2.0**-11 + 2.0**-20, 1.0 + 3 * 2.0**-11, 1.0 + 2.0**-8, 1.0 + 3 * 2.0**-8],
                 np.float32),
    ]
    # exact ties of both formats
    base = rng.integers(0, 2**15, 5000).astype(np.uint16)
    for dt, bit in (("f16", 12), ("bf16", 15)):
        f = decode64(base, dt).astype(np.float32)
        f = f[np.isfinite(f)]
        parts.append((f.view(np.uint32) | np.uint32(1 << bit)).view(np.float32))
    return np.concatenate(parts)


def test_encode_f16_matches_numpy_rne():
    f = _edge_floats()
    got = oracle.encode(f, "f16")
    with np.errstate(over="ignore", invalid="ignore"):
        want = f.astype(np.float16).view(np.uint16)
    nan = np.isnan(f)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7C00) == 0x7C00) and np.all((got[nan] & 0x3FF) != 0)


def test_encode_bf16_matches_torch_rne():
    f = _edge_floats()
    got = oracle.encode(f, "bf16")
    want = torch.from_numpy(f.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    nan = np.isnan(f)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.all((got[nan] & 0x7F80) == 0x7F80) and np.all((got[nan] & 0x7F) != 0)


def test_workload_encoder_agrees_with_oracle_encoder():
    # the generator's encoder and the oracle's are written separately
    f = _edge_floats()
    f = f[np.isfinite(f)]
    for dt in DTYPES:
        with np.errstate(over="ignore"):
            assert np.array_equal(wl.encode(f, dt), oracle.encode(f, dt))


# ------------------------------------------------------- defining equation
def _assert_matches_exact(y_bits, exact64, dtype, frac_equal=0.995, acc_rel=0.0):
    """y_bits must be the 16-bit rounding of exact64 up to accumulation noise."""
    got = decode64(y_bits, dtype)
    u = ulp(y_bits, dtype)
    err = np.abs(got - exact64)
    # half an ulp from the single rounding, plus accumulation error of the sums
    assert np.all(err <= 0.5 * u * (1 + 1e-9) + acc_rel * (1.0 + np.abs(exact64))), \
        float(np.max(err / u))
    want_bits = oracle.encode(exact64.astype(np.float32), dtype)  # double rounding is rare
    assert np.mean(want_bits == y_bits) >= frac_equal


@pytest.mark.parametrize("dtype", DTYPES)
def test_brute_force_tiny_config(dtype):
    w = wl.tiny(seed=0, dtype=dtype)
    exact = brute_force_add_lora(w)
    _assert_matches_exact(oracle.run_workload(w, acc64=True), exact, dtype, acc_rel=1e-12)
    _assert_matches_exact(oracle.run_workload(w, acc64=False), exact, dtype, acc_rel=2e-6,
                          frac_equal=0.98)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_brute_force_small_ragged(dtype, seed):
    # h=8, r=2, 5 tokens; plus odd sizes, an empty segment and a shared adapter
    w = wl.custom([2, 0, 3], 8, 8, 2, dtype, seed=seed, seg_adapter=[1, 0, 1], num_layers=2)
    for layer in (0, 1):
        exact = brute_force_add_lora(w, layer)
        _assert_matches_exact(oracle.run_workload(w, layer_idx=layer, acc64=True), exact, dtype,
                              acc_rel=1e-12, frac_equal=0.97)
    w = wl.custom([1, 4, 2, 5], 24, 40, 4, dtype, seed=seed, scale=0.5)
    exact = brute_force_add_lora(w)
    _assert_matches_exact(oracle.run_workload(w, acc64=True), exact, dtype, acc_rel=1e-12)
    _assert_matches_exact(oracle.run_workload(w, acc64=False), exact, dtype, acc_rel=2e-6,
                          frac_equal=0.98)


def test_non_square_shapes_catch_transposed_operands():
    # h_in != h_out != r: a transposed A or B indexes out of pattern and fails
    w = wl.custom([3, 2], 16, 48, 8, "f16", seed=5, num_layers=3)
    for layer in range(3):
        exact = brute_force_add_lora(w, layer)
        _assert_matches_exact(oracle.run_workload(w, layer_idx=layer, acc64=True), exact, "f16",
                              acc_rel=1e-12, frac_equal=0.97)


# ------------------------------------------------ special cases -> library
@pytest.mark.parametrize("dtype", DTYPES)
def test_identical_is_one_dense_product(dtype):
    w = wl.popularity("identical", batch=16, h_in=512, h_out=384, r=16, dtype=dtype,
                      num_layers=2, seed=3, scale=0.75)
    assert w.n_segs == 1
    x = decode64(w.x, dtype)
    A = decode64(w.A[0][1], dtype)
    B = decode64(w.B[0][1], dtype)
    exact = decode64(w.y0, dtype) + w.scale * np.matmul(np.matmul(x, A), B)
    _assert_matches_exact(oracle.run_workload(w, layer_idx=1, acc64=True), exact, dtype,
                          acc_rel=1e-12)
    _assert_matches_exact(oracle.run_workload(w, layer_idx=1, acc64=False), exact, dtype,
                          acc_rel=3e-6, frac_equal=0.98)


@pytest.mark.parametrize("dtype", DTYPES)
def test_distinct_is_gemv_per_token(dtype):
    w = wl.decode_distinct(batch=6, h_in=256, h_out=128, r=8, dtype=dtype, num_layers=1, seed=4)
    got = oracle.run_workload(w, acc64=True)
    for t in range(6):
        xt = decode64(w.x[t], dtype)
        vt = xt @ decode64(w.A[t][0], dtype)                 # vector-matrix, token's own pair
        exact = decode64(w.y0[t], dtype) + vt @ decode64(w.B[t][0], dtype)
        _assert_matches_exact(got[t], exact, dtype, acc_rel=1e-12, frac_equal=0.97)


def test_shrink_and_expand_separately_match_matmul():
    w = wl.custom([3, 5], 64, 96, 8, "f16", seed=9)
    v = oracle.run_workload(w, op="shrink", acc64=True)
    x = decode64(w.x, "f16")
    for i, (lo, hi) in enumerate([(0, 3), (3, 8)]):
        want = x[lo:hi] @ decode64(w.A[i][0], "f16")
        assert np.allclose(v[lo:hi], want, rtol=1e-6, atol=1e-6)
    # v += : accumulates on top of what is there
    v0 = np.full((8, 8), 2.5, np.float32)
    v2 = oracle.run_workload(w, op="shrink", acc64=True, v=v0)
    assert np.allclose(v2, v + 2.5, rtol=1e-6, atol=1e-6)
    # expand from a given v
    vin = np.random.Generator(np.random.PCG64(1)).standard_normal((8, 8)).astype(np.float32)
    y = oracle.run_workload(w, op="expand", v=vin, acc64=True)
    for i, (lo, hi) in enumerate([(0, 3), (3, 8)]):
        exact = decode64(w.y0[lo:hi], "f16") + vin[lo:hi].astype(np.float64) @ decode64(w.B[i][0], "f16")
        _assert_matches_exact(y[lo:hi], exact, "f16", acc_rel=1e-12, frac_equal=0.97)


# -------------------------------------------------------------- invariances
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("acc64", [False, True])
def test_two_launch_decomposition_equals_add_lora(dtype, acc64):
    w = wl.custom([2, 1, 4], 128, 64, 16, dtype, seed=6, scale=1.25)
    fused = oracle.run_workload(w, acc64=acc64)
    v = oracle.run_workload(w, op="shrink", acc64=acc64)
    two = oracle.run_workload(w, op="expand", v=v, acc64=acc64)
    if not acc64:
        assert np.array_equal(fused, two)          # same fp32 operations in the same order
    else:
        d = np.abs(fused.astype(np.int32) - two.astype(np.int32))
        assert d.max() <= 1 and np.mean(d == 0) > 0.99   # v passes through fp32 once


def test_permutation_invariance():
    # move whole segments (rows and adapter together): output rows move the same way
    lens = [2, 3, 1, 4]
    w = wl.custom(lens, 64, 64, 8, "f16", seed=7)
    y = oracle.run_workload(w)
    perm = [2, 0, 3, 1]
    starts = w.seg_starts
    rows = np.concatenate([np.arange(starts[p], starts[p + 1]) for p in perm])
    w2 = wl.custom([lens[p] for p in perm], 64, 64, 8, "f16", seed=7)
    w2.x, w2.y0 = w.x[rows].copy(), w.y0[rows].copy()
    w2.A, w2.B = w.A, w.B
    w2.seg_adapter = np.asarray(perm, np.int64)
    y2 = oracle.run_workload(w2)
    assert np.array_equal(y2, y[rows])


def test_segment_split_invariance():
    w = wl.custom([6, 2], 64, 64, 8, "bf16", seed=8)
    y = oracle.run_workload(w)
    w2 = wl.custom([1, 5, 2], 64, 64, 8, "bf16", seed=8, seg_adapter=[0, 0, 1])
    w2.x, w2.y0, w2.A, w2.B = w.x, w.y0, w.A, w.B
    assert np.array_equal(oracle.run_workload(w2), y)


def test_swapping_adapters_changes_the_result():
    # guards against an oracle that ignores the per-segment pointer
    w = wl.custom([2, 2], 64, 64, 8, "f16", seed=10)
    y = oracle.run_workload(w)
    w.seg_adapter = np.asarray([1, 0], np.int64)
    assert not np.array_equal(oracle.run_workload(w), y)


# ----------------------------------------------------------- exact routing
@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("acc64", [False, True])
def test_fingerprint_routing_is_bit_exact(dtype, acc64):
    lens = [1, 0, 3, 2, 0, 0, 5, 1]
    L = 3
    w = wl.fingerprint(lens, 32, 24, 8, dtype, num_layers=L)
    for layer in range(L):
        y = decode64(oracle.run_workload(w, layer_idx=layer, acc64=acc64), dtype)
        row = 0
        for a, n in enumerate(lens):
            for _ in range(n):
                assert np.all(y[row] == a + 1 + 32 * layer), (row, a, layer, y[row][:4])
                row += 1


def test_layer_offset_equals_presliced_weights():
    w = wl.custom([2, 3], 32, 48, 4, "f16", seed=12, num_layers=4)
    y = oracle.run_workload(w, layer_idx=2)
    w1 = wl.custom([2, 3], 32, 48, 4, "f16", seed=12, num_layers=4)
    w1.A = [np.ascontiguousarray(a[2:3]) for a in w.A]
    w1.B = [np.ascontiguousarray(b[2:3]) for b in w.B]
    w1.num_layers = 1
    assert np.array_equal(oracle.run_workload(w1, layer_idx=0), y)
    assert not np.array_equal(oracle.run_workload(w, layer_idx=1), y)


# ---------------------------------------------------------------- linearity
@pytest.mark.parametrize("dtype", DTYPES)
def test_zero_scale_and_zero_weights_leave_y_untouched(dtype):
    w = wl.custom([3, 2], 64, 64, 8, dtype, seed=13)
    w.scale = 0.0
    assert np.array_equal(oracle.run_workload(w), w.y0)
    w.scale = 1.0
    keepA = w.A
    w.A = [np.zeros_like(a) for a in w.A]
    assert np.array_equal(oracle.run_workload(w), w.y0)
    w.A = keepA
    w.B = [np.zeros_like(b) for b in w.B]
    assert np.array_equal(oracle.run_workload(w), w.y0)


def test_scale_doubles_the_addon():
    # y0 = 0 and power-of-two scales: Delta(2s) = 2 Delta(s) exactly, before and after rounding
    w = wl.custom([4, 4], 64, 64, 8, "f16", seed=14)
    w.y0 = np.zeros_like(w.y0)
    w.scale = 0.5
    y1 = decode64(oracle.run_workload(w), "f16")
    w.scale = 1.0
    y2 = decode64(oracle.run_workload(w), "f16")
    normal = np.abs(y1) >= 2.0 ** -13
    assert np.array_equal(y2[normal], 2 * y1[normal])


def test_sign_of_the_addon():
    # x = +1 on one feature, A, B positive  =>  y must increase
    w = wl.fingerprint([2], 16, 16, 8, "f16")
    w.y0 = wl.encode(np.full((2, 16), -3.0, np.float32), "f16")
    y = decode64(oracle.run_workload(w), "f16")
    assert np.all(y == -2.0)


# ---------------------------------------------------------------- edge cases
def test_null_pointer_segment_is_skipped_and_empty_inputs():
    w = wl.custom([2, 3, 1], 32, 32, 8, "f16", seed=15)
    full = oracle.run_workload(w)
    w.seg_adapter = np.asarray([0, -1, 2], np.int64)
    y = oracle.run_workload(w)
    assert np.array_equal(y[2:5], w.y0[2:5])
    assert np.array_equal(y[:2], full[:2]) and np.array_equal(y[5:], full[5:])
    # no segments at all
    empty = wl.custom([], 32, 32, 8, "f16", seed=15)
    assert oracle.run_workload(empty).shape == (0, 32)


@pytest.mark.parametrize("threads", [2, 3, 8])
def test_threads_do_not_change_a_bit(threads):
    w = wl.custom([5, 1, 7, 0, 4], 128, 96, 16, "bf16", seed=16)
    assert np.array_equal(oracle.run_workload(w, n_threads=threads), oracle.run_workload(w))
    v1 = oracle.run_workload(w, op="shrink", n_threads=threads)
    assert np.array_equal(v1, oracle.run_workload(w, op="shrink"))


def test_fp32_and_fp64_accumulation_agree_within_rounding():
    # bounds the oracle's own accumulation error at the metric width
    w = wl.decode_distinct(batch=4, h_in=4096, r=16, dtype="f16", num_layers=1, seed=17)
    y32 = oracle.run_workload(w, acc64=False)
    y64 = oracle.run_workload(w, acc64=True)
    a, b = decode64(y32, "f16"), decode64(y64, "f16")
    # fp32 sums of 4096 terms of size ~1/64 carry ~1e-6 of absolute error; on top
    # of that the two may round to neighbouring 16-bit values
    assert np.all(np.abs(a - b) <= ulp(y64, "f16") + 2e-5)
    assert np.mean(y32 == y64) > 0.97


# ------------------------------------------- single rounding of the fp64 variant
def _round16_exact(value, dtype):
    """Round an exact rational to the 16-bit format, nearest-even, by comparing it with
    the format's own values (numpy float16 / the upper half of a binary32)."""
    from fractions import Fraction
    if dtype == "f16":
        cands = np.arange(0x0000, 0x7C00, dtype=np.uint32).astype(np.uint16)   # finite, >= 0
    else:
        cands = np.arange(0x0000, 0x7F80, dtype=np.uint32).astype(np.uint16)
    vals = decode64(cands, dtype)
    sign = 0x8000 if value < 0 else 0
    mag = abs(value)
    hi = int(np.searchsorted(vals, float(mag), side="left"))
    hi = min(max(hi, 1), len(vals) - 1)
    best = None
    for i in (hi - 1, hi, min(hi + 1, len(vals) - 1)):
        err = abs(Fraction(float(vals[i])) - mag)
        key = (err, int(cands[i]) & 1)            # nearest, then even significand
        if best is None or key < best[0]:
            best = (key, int(cands[i]))
    return best[1] | sign


@pytest.mark.parametrize("dtype", DTYPES)
def test_fp64_variant_rounds_once_across_16_bit_ties(dtype):
    # y + v.B built so that the exact sum sits a hair (2^-40) above or below a tie of the
    # 16-bit format, or exactly on it.  Rounding the fp64 sum to fp32 first and then to 16
    # bits lands on the tie and picks the wrong neighbour; one rounding does not.
    from fractions import Fraction
    half_ulp = Fraction(1, 2 ** 11) if dtype == "f16" else Fraction(1, 2 ** 8)   # at 1.0
    tiny = Fraction(1, 2 ** 40)
    cases = []
    for sgn in (1, -1):
        for odd_multiple in (1, 3, 5):
            for nudge in (tiny, -tiny, 0):
                cases.append((sgn, odd_multiple, nudge))
    T, r = len(cases), 8
    one = {"f16": 0x3C00, "bf16": 0x3F80}[dtype]
    B = np.zeros((1, r, 8), np.uint16)
    B[0, :, :] = one                                   # every B entry is 1.0
    y0 = np.zeros((T, 8), np.uint16)
    v = np.zeros((T, r), np.float32)
    want = np.zeros((T, 8), np.uint16)
    for t, (sgn, m, nudge) in enumerate(cases):
        y0[t, :] = one | (0x8000 if sgn < 0 else 0)    # +-1.0
        v[t, 0] = sgn * float(m * half_ulp)            # exact in fp32
        v[t, 1] = sgn * float(nudge)                   # +-2^-40 or 0, exact in fp32
        exact = sgn * (1 + m * half_ulp + nudge)
        want[t, :] = _round16_exact(exact, dtype)
    got = oracle.expand(dtype, y0.copy(), v, [B], [0, T], acc64=True)
    assert np.array_equal(got, want)
    # the nudged cases really are ones where two roundings go wrong
    twice = wl.encode((decode64(y0, dtype)[:, 0] + v.astype(np.float64).sum(axis=1)).astype(np.float32), dtype)
    assert np.any(twice != want[:, 0])


# ------------------------------------------- fp32 "v +=" on top of what is there
def test_fp32_shrink_adds_into_nonzero_v_with_one_fp32_addition():
    # small integers: x.A is exact in fp32 whatever the order, so v0 + x.A has one rounding
    rng = np.random.Generator(np.random.PCG64(31))
    T, h_in, r = 7, 48, 8
    xi = rng.integers(-3, 4, (T, h_in)).astype(np.float32)
    Ai = rng.integers(-3, 4, (2, 1, h_in, r)).astype(np.float32)
    x = wl.encode(xi, "f16")
    A = [wl.encode(Ai[0], "f16"), wl.encode(Ai[1], "f16")]
    starts = [0, 3, 7]
    prod = np.concatenate([xi[:3].astype(np.int64) @ Ai[0, 0].astype(np.int64),
                           xi[3:].astype(np.int64) @ Ai[1, 0].astype(np.int64)])
    # starting values: fractions, a negative, and 2^24 (+3 is then inexact in fp32: ties to even)
    v0 = np.tile(np.asarray([1.5, -2.25, 0.0, 16777216.0, -16777216.0, 1e-3, 3.0e7, -0.5], np.float32), (T, 1))
    got = oracle.shrink("f16", v0.copy(), x, A, starts, acc64=False)
    want = v0 + prod.astype(np.float32)                # numpy's fp32 addition, one rounding
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert not np.array_equal(got, prod.astype(np.float32))          # it did add, not overwrite
    # a second call accumulates again
    got2 = oracle.shrink("f16", got.copy(), x, A, starts, acc64=False)
    assert np.array_equal(got2.view(np.uint32), (want + prod.astype(np.float32)).view(np.uint32))
