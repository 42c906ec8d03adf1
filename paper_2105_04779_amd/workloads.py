"""Seeded synthetic inputs for the EL-attention decode step.

This module holds no arithmetic of the method: it only draws random tensors
with the shapes, value distributions and length mixes of the workloads, rounds
them once to the storage dtype, and hands the identical values to whoever asks
(the HIP path, the CPU oracle's tests, the benchmark).

Recipe (every workload):
  H, queries  ~ N(0, 1)
  W_q, W_k, W_v, W_o ~ N(0, 1/d_m)   (standard deviation d_m**-0.5)
  b_q, b_k, b_v, b_o ~ N(0, 0.02**2) (standard deviation 0.02)
  lengths     ~ uniform integers in [len_lo, len_hi]
All values are drawn in float32 from numpy's PCG64 and rounded to nearest-even
to the storage dtype once; the rounded values (as float32) are what both sides
receive.  Every batch element has its own stream, so any subset of a large
workload can be regenerated without drawing the rest.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 210504779

# stream identifiers inside one workload's seed sequence
_S_WEIGHTS, _S_LENGTHS, _S_ELEMENT = 1, 2, 3


@dataclass(frozen=True)
class Workload:
    name: str
    index: int          # position in the benchmark's list of configurations
    dtype: str          # storage dtype of H, queries and weights: "f32" | "f16" | "bf16"
    B: int              # number of distinct hidden-state matrices
    beam: int           # queries sharing one H
    heads: int
    d_m: int
    d_k: int
    n: int              # padded key length
    len_lo: int
    len_hi: int
    note: str = ""

    @property
    def R(self) -> int:
        """Expanded-query rows that share one H (heads x beam)."""
        return self.heads * self.beam

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


WORKLOADS = {
    w.name: w
    for w in [
        Workload("c1_tiny_f32", 0, "f32", 2, 2, 4, 64, 16, 32, 32, 32,
                 "tiny fp32 cross-attention"),
        Workload("c2_transformer_base_f16", 1, "f16", 64, 4, 8, 512, 64, 512, 256, 512,
                 "Transformer-base-shaped fp16 cross-attention"),
        Workload("c3_bart_large_bf16", 2, "bf16", 64, 4, 16, 1024, 64, 1024, 512, 1024,
                 "BART-large-shaped bf16 beam-search cross-attention"),
        Workload("c4_bart_large_b320_bf16", 3, "bf16", 320, 4, 16, 1024, 64, 1024, 512, 1024,
                 "BART-large shape at batch 320"),
        # GPT-2-medium self-attention: batch 128 x beam 4 with a per-beam history,
        # i.e. 512 independent H matrices with one query each, all of length n.
        Workload("c5_gpt2_medium_n512_bf16", 4, "bf16", 512, 1, 16, 1024, 64, 512, 512, 512,
                 "GPT-2-medium-shaped self-attention, history 512"),
        Workload("c5_gpt2_medium_n768_bf16", 4, "bf16", 512, 1, 16, 1024, 64, 768, 768, 768,
                 "GPT-2-medium-shaped self-attention, history 768"),
        Workload("c5_gpt2_medium_n1024_bf16", 4, "bf16", 512, 1, 16, 1024, 64, 1024, 1024, 1024,
                 "GPT-2-medium-shaped self-attention, history 1024"),
    ]
}


def custom(name="custom", *, dtype, B, beam, heads, d_m, d_k, n, len_lo=None, len_hi=None, index=99):
    """A workload of arbitrary shape with the same recipe (tests use this)."""
    return Workload(name, index, dtype, B, beam, heads, d_m, d_k, n,
                    n if len_lo is None else len_lo, n if len_hi is None else len_hi)


def with_batch(w: Workload, B: int) -> Workload:
    return replace(w, B=B)


# ---------------------------------------------------------------------------------------------
# rounding to the storage dtype (representation only, no method arithmetic)
# ---------------------------------------------------------------------------------------------
def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to nearest-even in `dtype`; return them as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32)
        bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
        r = (u + bias) & np.uint32(0xFFFF0000)
        nan = np.isnan(x)
        if nan.any():
            r = np.where(nan, np.uint32(0x7FC00000), r)
        return r.view(np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Bit pattern of already-rounded float32 values in the storage dtype.

    f32 -> float32 array, f16 -> float16 array, bf16 -> uint16 array (upper halves).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype!r}")


def _rng(w: Workload, *stream) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED, w.index, *stream])))


# ---------------------------------------------------------------------------------------------
# generators
# ---------------------------------------------------------------------------------------------
def weights(w: Workload) -> dict:
    """W_q, W_k, W_v [d_m, h*d_k], W_o [h*d_k, d_m], b_q, b_k, b_v [h*d_k], b_o [d_m]."""
    g = _rng(w, _S_WEIGHTS)
    hd = w.heads * w.d_k
    std = float(w.d_m) ** -0.5
    out = {}
    for name, shape in (("Wq", (w.d_m, hd)), ("Wk", (w.d_m, hd)), ("Wv", (w.d_m, hd)), ("Wo", (hd, w.d_m))):
        out[name] = round_to_storage(g.standard_normal(shape, dtype=np.float32) * np.float32(std), w.dtype)
    for name, size in (("bq", hd), ("bk", hd), ("bv", hd), ("bo", w.d_m)):
        out[name] = round_to_storage(g.standard_normal(size, dtype=np.float32) * np.float32(0.02), w.dtype)
    return out


def lengths(w: Workload) -> np.ndarray:
    """Valid-prefix length of every batch element, int32 [B], in [len_lo, len_hi]."""
    g = _rng(w, _S_LENGTHS)
    return g.integers(w.len_lo, w.len_hi, size=w.B, endpoint=True).astype(np.int32)


def batch_element(w: Workload, b: int, length: int | None = None, poison: bool = False):
    """(H_b [n, d_m], queries_b [beam, d_m]) of batch element b, rounded, as float32.

    With `poison`, rows at and beyond `length` are NaN (they must never be read);
    otherwise they hold finite noise like the valid rows.
    """
    g = _rng(w, _S_ELEMENT, b)
    Hb = round_to_storage(g.standard_normal((w.n, w.d_m), dtype=np.float32), w.dtype)
    qb = round_to_storage(g.standard_normal((w.beam, w.d_m), dtype=np.float32), w.dtype)
    if poison and length is not None and length < w.n:
        Hb[length:, :] = np.nan
    return Hb, qb


def batch(w: Workload, elements=None, poison: bool = False):
    """Stack batch elements (all of them, or the listed ones).

    Returns (H [k, n, d_m], queries [k, beam, d_m], lengths [k]) as float32/int32.
    """
    lens = lengths(w)
    idx = list(range(w.B)) if elements is None else list(elements)
    H = np.empty((len(idx), w.n, w.d_m), dtype=np.float32)
    Q = np.empty((len(idx), w.beam, w.d_m), dtype=np.float32)
    for k, b in enumerate(idx):
        H[k], Q[k] = batch_element(w, b, int(lens[b]), poison)
    return H, Q, lens[idx].copy()
