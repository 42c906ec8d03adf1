"""Closed-form byte and flop counts for the attention decode step (host logic).

Used by the benchmark to turn a measured time into roofline fractions, and
pinned in the CPU tests to the counts the paper prints (Table 4, section 4.1.1).
Symbols follow the paper: B batch, x beam, h heads, d_m model width, d_k head
width, n key length, L decoder layers.
"""
from __future__ import annotations

GiB = float(1 << 30)


def el_state_bytes(B: int, n: int, d_m: int, elem_bytes: int = 2) -> int:
    """Input-related state EL-attention keeps: the encoder output, once (section 3.1.1)."""
    return B * n * d_m * elem_bytes


def mha_cache_bytes(B: int, n: int, d_m: int, layers: int, beam: int, elem_bytes: int = 2) -> int:
    """Per-layer key and value caches of multi-head attention, repeated per beam (Table 4)."""
    return 2 * layers * beam * el_state_bytes(B, n, d_m, elem_bytes)


def build_kv_flops(B: int, beam: int, n: int, d_m: int) -> int:
    """Group 1 of Table 1 without a cache: project K and V for every beam's copy of H."""
    return 2 * 2 * (B * beam * n) * d_m * d_m


def mha_group3_bytes(B: int, beam: int, n: int, d_m: int, elem_bytes: int = 2) -> int:
    """Group 3 with cached multi-head K and V: both are read once per beam (O(x n d_m))."""
    return 2 * B * beam * n * d_m * elem_bytes


def el_group3_bytes_two_reads(B: int, n: int, d_m: int, elem_bytes: int = 2) -> int:
    """Group 3 with EL-attention as two library calls: H is read by the score
    product and again by the weighted sum (O(n d_m), no beam factor)."""
    return 2 * B * n * d_m * elem_bytes


def step_algorithmic_bytes(sum_len: int, B: int, beam: int, d_m: int, hd: int,
                           elem_bytes: int, out_bytes: int = 4) -> int:
    """Bytes one fused decode step has to move: the valid rows of H once, the four
    weight matrices, the queries and the output.  Intermediates are not credited."""
    return (sum_len * d_m * elem_bytes + (3 * d_m * hd + hd * d_m) * elem_bytes
            + B * beam * d_m * (elem_bytes + out_bytes))


def core_algorithmic_bytes(sum_len: int, d_m: int, elem_bytes: int) -> int:
    """Bytes the attention-core kernel has to read: the valid rows of H, once."""
    return sum_len * d_m * elem_bytes


def step_flops(sum_len: int, B: int, beam: int, heads: int, d_m: int, d_k: int) -> int:
    """Scores + weighted sum over H for all h*x rows, plus the four small projections."""
    R = heads * beam
    hd = heads * d_k
    core = 4 * R * sum_len * d_m
    proj = 2 * B * beam * d_m * hd * 2 + 2 * B * beam * heads * d_k * d_m * 2
    return core + proj


def core_flops(sum_len: int, beam: int, heads: int, d_m: int) -> int:
    return 4 * heads * beam * sum_len * d_m
