"""Literal fp64 definitions (dense S x S matrices).  TEST INFRASTRUCTURE ONLY.

Every function works on one batch element.  Attention tensors are laid out
``[S, H, D]`` (full sequence, this device's heads, head dim), the layout a
device holds inside the attention layer of a Ulysses-style step (Section 2,
Figure 1 caption: attention layers see the whole sequence but a subset of the
heads).  Query head ``a`` reads key/value head ``a // G`` with
``G = Hq // Hkv`` (the evaluated models use grouped-query or full attention,
Section 4 setup).  The mask is causal, diagonal included (Section 3.1,
challenge 3 names the causal mask as part of the model).

Readings taken where the paper is silent: natural-log LSE that includes the
softmax scale; default scale 1/sqrt(D); contiguous head grouping.

Pinned by tests/test_oracle_pins.py (brute force, closed forms, invariants,
finite differences, simulated P-rank equivalence).
"""
from __future__ import annotations

import numpy as np


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> fp64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# Re-layout around the all-to-all (Section 2: the all-to-all re-shards the
# activations from the sequence dimension to the head dimension and back).
# Input  [S_l, H, D]   : this rank's S_l = S/P tokens, all H heads.
# Output [P*S_l, h, D] : h = H/P; rows p*S_l .. (p+1)*S_l-1 are the chunk that
#                        goes to rank p (its heads p*h .. p*h+h-1).
# --------------------------------------------------------------------------
def pack_seq_to_head(x: np.ndarray, P: int) -> np.ndarray:
    S_l, H, D = x.shape
    assert H % P == 0
    h = H // P
    return np.ascontiguousarray(x.reshape(S_l, P, h, D).transpose(1, 0, 2, 3)).reshape(P * S_l, h, D)


def unpack_head_to_seq(y: np.ndarray, P: int) -> np.ndarray:
    PS, h, D = y.shape
    assert PS % P == 0
    S_l = PS // P
    return np.ascontiguousarray(y.reshape(P, S_l, h, D).transpose(1, 0, 2, 3)).reshape(S_l, P * h, D)


def pack_seq_to_head_loops(x: np.ndarray, P: int) -> np.ndarray:
    """Same map written as explicit index loops: out[p*S_l+s, j] = in[s, p*h+j]."""
    S_l, H, D = x.shape
    h = H // P
    out = np.empty((P * S_l, h, D), dtype=x.dtype)
    for p in range(P):
        for s in range(S_l):
            for j in range(h):
                out[p * S_l + s, j, :] = x[s, p * h + j, :]
    return out


def unpack_head_to_seq_loops(y: np.ndarray, P: int) -> np.ndarray:
    PS, h, D = y.shape
    S_l = PS // P
    out = np.empty((S_l, P * h, D), dtype=y.dtype)
    for p in range(P):
        for s in range(S_l):
            for j in range(h):
                out[s, p * h + j, :] = y[p * S_l + s, j, :]
    return out


# --------------------------------------------------------------------------
# Causal grouped-query attention, dense.
# --------------------------------------------------------------------------
def _scale(D: int, softmax_scale) -> float:
    return float(softmax_scale) if (softmax_scale is not None and softmax_scale > 0) else 1.0 / np.sqrt(D)


def _probabilities(qa: np.ndarray, kg: np.ndarray, scale: float):
    """Scores, LSE and softmax matrix of one head: qa [S,D], kg [S,D]."""
    S = qa.shape[0]
    s = scale * (qa @ kg.T)                                   # s_ij
    s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)  # j > i masked
    m = s.max(axis=1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(s - m).sum(axis=1))
    p = np.exp(s - lse[:, None])
    return p, lse


def attn_fwd(q, k, v, softmax_scale=None):
    """q [S,Hq,D], k,v [S,Hkv,D] fp64 -> O [S,Hq,D], LSE [Hq,S]."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    S, Hq, D = q.shape
    Hkv = k.shape[1]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    scale = _scale(D, softmax_scale)
    o = np.empty((S, Hq, D))
    lse = np.empty((Hq, S))
    for a in range(Hq):
        g = a // G
        p, lse[a] = _probabilities(q[:, a], k[:, g], scale)
        o[:, a] = p @ v[:, g]
    return o, lse


def attn_bwd(q, k, v, do, softmax_scale=None):
    """Gradient of L = sum(O * dO) w.r.t. q, k, v.  Returns dQ, dK, dV, Delta[Hq,S]."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64); do = np.asarray(do, np.float64)
    S, Hq, D = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    scale = _scale(D, softmax_scale)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    delta = np.empty((Hq, S))
    for a in range(Hq):
        g = a // G
        p, _ = _probabilities(q[:, a], k[:, g], scale)
        o = p @ v[:, g]
        delta[a] = (do[:, a] * o).sum(axis=1)                 # Delta_i = dO_i . O_i
        dp = do[:, a] @ v[:, g].T                             # dP_ij = dO_i . v_j
        ds = p * (dp - delta[a][:, None])                     # dS_ij
        dq[:, a] = scale * (ds @ k[:, g])
        dk[:, g] += scale * (ds.T @ q[:, a])
        dv[:, g] += p.T @ do[:, a]
    return dq, dk, dv, delta


# --------------------------------------------------------------------------
# Packed documents: rows [cu[t], cu[t+1]) form document t; a query sees the
# keys of its own document at or before its own position.  Not in the paper;
# it is the block-diagonal version of the same operator.
# --------------------------------------------------------------------------
def attn_varlen_fwd(q, k, v, cu_seqlens, softmax_scale=None):
    T, Hq, D = q.shape
    o = np.zeros((T, Hq, D)); lse = np.zeros((Hq, T))
    cu = [int(c) for c in cu_seqlens]
    for t in range(len(cu) - 1):
        a, b = cu[t], cu[t + 1]
        if b > a:
            o[a:b], lse[:, a:b] = attn_fwd(q[a:b], k[a:b], v[a:b], _scale(D, softmax_scale))
    return o, lse


def attn_varlen_bwd(q, k, v, do, cu_seqlens, softmax_scale=None):
    T, Hq, D = q.shape
    dq = np.zeros((T, Hq, D)); dk = np.zeros(k.shape); dv = np.zeros(v.shape)
    delta = np.zeros((Hq, T))
    cu = [int(c) for c in cu_seqlens]
    for t in range(len(cu) - 1):
        a, b = cu[t], cu[t + 1]
        if b > a:
            dq[a:b], dk[a:b], dv[a:b], delta[:, a:b] = attn_bwd(
                q[a:b], k[a:b], v[a:b], do[a:b], _scale(D, softmax_scale))
    return dq, dk, dv, delta
