"""Byte and flop accounting of SGMV (host arithmetic for the benchmark's roofline).

``paper_io_bytes`` / ``paper_flop`` are the closed forms of the paper's roofline
paragraph (FLOP = s_n * h_i * h_o * 2, I/O = [s_n (h_i + h_o) + n h_i h_o] * 2 for
one SGMV launch with 16-bit data).  ``algorithmic_bytes`` is the finer count
this build reports against: it also counts that expand reads *and* writes y and
that v is fp32.
"""
from __future__ import annotations

E = 2  # bytes per 16-bit element


def paper_flop(s_n: int, h_i: int, h_o: int) -> int:
    return s_n * h_i * h_o * 2


def paper_io_bytes(s_n: int, n: int, h_i: int, h_o: int) -> int:
    return (s_n * (h_i + h_o) + n * h_i * h_o) * 2


def shrink_bytes(T: int, n: int, h_in: int, r: int) -> int:
    """weights of the n distinct adapters + x read + v (fp32) written"""
    return n * h_in * r * E + T * h_in * E + T * r * 4


def expand_bytes(T: int, n: int, r: int, h_out: int) -> int:
    """weights + v (fp32) read + y read and written"""
    return n * r * h_out * E + T * r * 4 + 2 * T * h_out * E


def algorithmic_bytes(op: str, T: int, n: int, h_in: int, h_out: int, r: int) -> int:
    if op == "shrink":
        return shrink_bytes(T, n, h_in, r)
    if op == "expand":
        return expand_bytes(T, n, r, h_out)
    if op == "add_lora":
        return shrink_bytes(T, n, h_in, r) + expand_bytes(T, n, r, h_out)
    raise ValueError(op)


def flops(op: str, T: int, h_in: int, h_out: int, r: int) -> int:
    s = 2 * T * h_in * r
    e = 2 * T * r * h_out
    return {"shrink": s, "expand": e, "add_lora": s + e}[op]
