"""Test-side helpers that are independent of both the oracle and the HIP path.

Decoding of 16-bit patterns uses numpy's own float16 and the definition of
bfloat16 (upper half of an IEEE binary32), so that the oracle's hand-written
conversions are checked against something other than themselves.
"""
import numpy as np


def decode64(bits: np.ndarray, dtype: str) -> np.ndarray:
    bits = np.ascontiguousarray(bits, np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def ulp(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Spacing of the 16-bit format at each value (float64)."""
    val = np.abs(decode64(bits, dtype))
    if dtype == "f16":
        mant, emin = 10, -14
    else:
        mant, emin = 7, -126
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(val > 0, val, 1.0)))
    e = np.maximum(e, emin)
    e = np.where(val > 0, e, emin)
    return np.power(2.0, e - mant)


def brute_force_add_lora(w, layer_idx=0):
    """Straight from the operator's defining equation, in fp64, token by token.

    Structurally different from the oracle on purpose: every token searches for
    its own segment, and the adapter's full h_in x h_out product A_i B_i is
    formed first, so the row result is x (A_i B_i) rather than (x A_i) B_i.
    Returns float64 [T, h_out] (unrounded).
    """
    T = w.n_tokens
    x = decode64(w.x, w.dtype)
    y = decode64(w.y0, w.dtype).copy()
    prod_cache = {}
    for t in range(T):
        seg = None
        for i in range(w.n_segs):           # linear search for the token's segment
            if w.seg_starts[i] <= t < w.seg_starts[i + 1]:
                seg = i
                break
        assert seg is not None
        a = int(w.seg_adapter[seg])
        if a < 0:
            continue
        if a not in prod_cache:
            Aa = decode64(w.A[a][layer_idx], w.dtype)
            Ba = decode64(w.B[a][layer_idx], w.dtype)
            prod_cache[a] = Aa @ Ba
        y[t] += w.scale * (x[t] @ prod_cache[a])
    return y


def tolerance(ref64: np.ndarray) -> np.ndarray:
    """The parity bar: |got - ref| <= 2e-3 + 2e-2 |ref|."""
    return 2e-3 + 2e-2 * np.abs(ref64)
