"""Seeded synthetic queries and keys shaped like the paper's workloads.

Input plumbing only: this module holds none of the method's arithmetic and is
the one piece of code that both the HIP path's tests/benchmark and the CPU
oracle's tests may use.  Everything is numpy on the host; values are drawn in
float32, cast ONCE to the storage dtype, and the cast values are the ground
truth for both sides.

The tensors stand in for the query/key activations of Llama-2-7B /
Llama-3.1-8B on LongBench-length prompts (Section 4 and the setup appendix of
the paper): only their shapes and two qualitative statistics are borrowed,
namely a few large-magnitude "outlier" channels in the keys (Related Work,
KV cache compression) and queries that concentrate in a low-dimensional
subspace (Section 3.2).
"""
from __future__ import annotations

import numpy as np

BF16 = "bf16"
F16 = "f16"
F32 = "f32"


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


# ---- storage dtypes ------------------------------------------------------- #

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def store(x32: np.ndarray, dtype: str):
    """Cast float32 draws to the storage dtype.

    Returns (raw, value): `raw` is what is handed to the library (float32 array,
    float16 array, or uint16 array of bf16 bit patterns), `value` the same
    numbers as float64 for the oracle.
    """
    if dtype == F32:
        raw = np.ascontiguousarray(x32, dtype=np.float32)
        return raw, raw.astype(np.float64)
    if dtype == F16:
        raw = np.ascontiguousarray(x32, dtype=np.float32).astype(np.float16)
        return raw, raw.astype(np.float64)
    if dtype == BF16:
        raw = f32_to_bf16_bits(x32)
        return raw, bf16_bits_to_f32(raw).astype(np.float64)
    raise ValueError(dtype)


# ---- distributions -------------------------------------------------------- #

def outlier_channels(gen: np.random.Generator, heads: int, d: int,
                     count=(2, 6), scale=(8.0, 15.0)):
    """Per head: a few channel indices and their magnification factors."""
    out = []
    for _ in range(heads):
        n = int(gen.integers(count[0], count[1] + 1))
        idx = gen.choice(d, size=n, replace=False)
        fac = gen.uniform(scale[0], scale[1], size=n).astype(np.float32)
        out.append((np.sort(idx), fac[np.argsort(idx)]))
    return out


def keys(seed: int, heads: int, n: int, d: int = 128, *, heavy_tail: bool = False,
         outliers=(2, 6), outlier_scale=(8.0, 15.0), batch: int | None = None) -> np.ndarray:
    """float32 keys [heads, n, d] (or [batch, heads, n, d]).

    N(0,1) per element (Student-t with 4 degrees of freedom per element if
    heavy_tail), then per head a few channels are multiplied by a factor.
    """
    gen = rng(seed)
    shape = (heads, n, d) if batch is None else (batch, heads, n, d)
    if heavy_tail:
        x = gen.standard_t(4.0, size=shape).astype(np.float32)
    else:
        x = gen.standard_normal(size=shape, dtype=np.float32)
    if outliers is not None and outliers[1] > 0:
        oc = outlier_channels(gen, heads, d, outliers, outlier_scale)
        for h, (idx, fac) in enumerate(oc):
            if batch is None:
                x[h][:, idx] *= fac
            else:
                x[:, h][..., idx] *= fac
    return x


def queries(seed: int, q_heads: int, n: int, d: int = 128, *,
            planted_rank: int = 0, planted_gain: float = 4.0) -> np.ndarray:
    """float32 prompt queries [q_heads, n, d].

    N(0,1); with planted_rank > 0 a random orthonormal set of that many
    directions per head is amplified by a decaying gain, so that the leading
    singular subspace is well separated (the "queries live in a small
    subspace" regime of Section 3.2).
    """
    gen = rng(seed)
    x = gen.standard_normal(size=(q_heads, n, d), dtype=np.float32)
    if planted_rank > 0:
        for h in range(q_heads):
            B, _ = np.linalg.qr(gen.standard_normal(size=(d, planted_rank)))
            gains = planted_gain * (0.85 ** np.arange(planted_rank))
            coef = x[h].astype(np.float64) @ B                 # (n, pr)
            x[h] += (coef * gains) @ B.T
    return x.astype(np.float32)
