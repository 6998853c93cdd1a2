"""Seeded synthetic inputs for the Ulysses-shard hot path.

This module holds no arithmetic of the method itself: it only draws random
numbers, rounds them to bf16 bit patterns and builds document-length lists.
It is the one module that both the CPU oracle's tests and the HIP path's
tests/bench draw inputs from, so that both sides see identical bits.

bf16 tensors are carried as numpy ``uint16`` arrays of bit patterns (numpy has
no bf16 dtype); every bf16 value is exactly representable in fp32 and fp64.

Shapes follow the per-GPU shard the paper's Ulysses description implies
(Section 2, Figure 1): outside attention a device holds ``[S/P, H, D]``
(partial sequence, all heads); inside attention ``[S, H/P, D]`` (full
sequence, its own heads).
"""
from __future__ import annotations

import math

import numpy as np

__all__ = [
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "normal_bf16",
    "attn_inputs",
    "pack_input",
    "doc_lengths",
    "cu_seqlens_from_lengths",
    "CONFIGS",
]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    r = ((u + bias) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to fp32 (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape, scale: float = 1.0) -> np.ndarray:
    """iid N(0, scale^2) drawn in fp32, rounded to bf16 bits."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x = x * np.float32(scale)
    return f32_to_bf16_bits(x)


def attn_inputs(seed: int, S: int, Hq: int, Hkv: int, D: int, B: int = 1):
    """Q, K, V, dO as bf16 bit arrays, independent streams per tensor.

    Layout ``[B, S, H, D]`` (head-sharded, full sequence), values iid N(0,1).
    """
    ss = np.random.SeedSequence([int(seed), 0x5EED])
    rq, rk, rv, rd = (np.random.default_rng(s) for s in ss.spawn(4))
    q = normal_bf16(rq, (B, S, Hq, D))
    k = normal_bf16(rk, (B, S, Hkv, D))
    v = normal_bf16(rv, (B, S, Hkv, D))
    do = normal_bf16(rd, (B, S, Hq, D))
    return q, k, v, do


def pack_input(seed: int, B: int, S_l: int, H: int, D: int, kind: str = "random") -> np.ndarray:
    """A ``[B, S_l, H, D]`` 16-bit tensor for the re-layout kernels.

    ``kind='iota'`` numbers the elements (mod 2^16) so every output element
    names its source; ``kind='random'`` draws uniform random bit patterns
    (all 2^16 patterns, including NaN/Inf encodings: the re-layout is a byte
    permutation and must carry them unchanged).
    """
    n = B * S_l * H * D
    if kind == "iota":
        return (np.arange(n, dtype=np.uint64) % 65521).astype(np.uint16).reshape(B, S_l, H, D)
    rng = np.random.default_rng([int(seed), 0xFACC])
    return rng.integers(0, 1 << 16, size=(B, S_l, H, D), dtype=np.uint16)


def doc_lengths(seed: int, total: int = 65536, mean: float = 4096.0, sigma: float = 1.0,
                lo: int = 128, hi: int = 32768) -> list[int]:
    """Document lengths for the packed variable-length workload.

    Lognormal whose *distribution mean* is ``mean`` (mu = ln(mean) - sigma^2/2),
    floor, clip to [lo, hi]; drawn until the running total reaches ``total``;
    the last document is cut to fit and merged into its predecessor if the cut
    leaves fewer than ``lo`` tokens.
    """
    rng = np.random.default_rng([int(seed), 0xD0C5])
    mu = math.log(mean) - 0.5 * sigma * sigma
    out: list[int] = []
    acc = 0
    while acc < total:
        L = int(min(max(math.floor(rng.lognormal(mu, sigma)), lo), hi))
        L = min(L, total - acc)
        out.append(L)
        acc += L
    if len(out) > 1 and out[-1] < lo:
        out[-2] += out[-1]
        out.pop()
    assert sum(out) == total
    return out


def cu_seqlens_from_lengths(lengths) -> np.ndarray:
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return cu


# The workloads named by the build's baseline file: one GPU's shard at P=8
# (P=4 for the tiny case).
CONFIGS = {
    "tiny": dict(S=512, Hq=2, Hkv=1, D=64, pack=dict(S_l=512, H=8, D=64, P=4)),
    "c2_8b_32k": dict(S=32768, Hq=4, Hkv=1, D=128, pack=dict(S_l=4096, H=32, D=128, P=8)),
    "c3_8b_128k": dict(S=131072, Hq=4, Hkv=1, D=128, pack=dict(S_l=16384, H=32, D=128, P=8)),
    "c4_70b_128k": dict(S=131072, Hq=8, Hkv=1, D=128, pack=dict(S_l=16384, H=64, D=128, P=8)),
    "c5_varlen_64k": dict(T=65536, Hq=4, Hkv=1, D=128),
}
