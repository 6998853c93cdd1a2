"""Blockwise attention step and the (O, LSE) merge, literal fp64 definitions.
TEST INFRASTRUCTURE ONLY.

The paper's second workload is the ring-style schedule it compares against
(Section 4, baselines; Section 4.1, runtime performance: keys and values are
exchanged around a ring in p steps): the sequence stays sharded, key/value
blocks travel from device to device, and a device combines the partial
attention of its query block against one key/value block at a time.  What one
device computes per arriving block is defined here, for one batch element:

* ``block_attn_fwd``: softmax attention of a query block [Sq,Hq,D] against a
  key/value block [Skv,Hkv,D] where query row i sees keys j <= i + off.  With
  the query block starting at global position a and the key block at global
  position c, causal attention over the whole sequence is off = a - c; any
  off >= Skv-1 hides nothing, off = 0 with equal blocks is the diagonal block.
  A row that sees no key has O = 0 and LSE = -inf.
* ``merge``: the softmax over the union of two disjoint key sets from the two
  partial results: LSE = log(e^LSE_a + e^LSE_b), O = the LSE-weighted mean.
* ``block_attn_bwd``: this block pair's share of the gradients of
  L = sum(O_final * dO), given the *final* (merged) LSE and
  Delta_i = dO_i . O_final_i of the query rows:
  P_ij = exp(scale q_i.k_j - LSE_i), dV_j += P_ij dO_i,
  dS_ij = P_ij (dO_i.v_j - Delta_i), dQ_i += scale dS_ij k_j, dK_j += scale dS_ij q_i.
  Summed over all key blocks (dQ) or all query blocks (dK, dV) the shares give
  the gradients of attention over the whole sequence.

Readings where the paper is silent (it names the schedule, not its arithmetic):
natural-log LSE that includes the softmax scale, grouped heads contiguous
(query head a reads key/value head a // G), mask boundary inclusive.

Pinned by tests/test_block_pins.py (scalar brute force, library softmax, the
unmasked and the diagonal special cases, union-of-key-sets identity, sums of
block shares against torch fp64 autograd of attention over the whole sequence).
"""
from __future__ import annotations

import numpy as np


def _visible(Sq: int, Skv: int, off: int) -> np.ndarray:
    i = np.arange(Sq)[:, None]
    j = np.arange(Skv)[None, :]
    return j <= i + off


def block_attn_fwd(q, k, v, scale: float, off: int):
    """q [Sq,Hq,D], k,v [Skv,Hkv,D] -> O [Sq,Hq,D], LSE [Hq,Sq]."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    Sq, Hq, D = q.shape
    Skv, Hkv, _ = k.shape
    assert Hq % Hkv == 0
    G = Hq // Hkv
    vis = _visible(Sq, Skv, off)
    o = np.zeros((Sq, Hq, D))
    lse = np.full((Hq, Sq), -np.inf)
    for a in range(Hq):
        g = a // G
        s = np.where(vis, scale * (q[:, a] @ k[:, g].T), -np.inf)
        m = s.max(axis=1)
        rows = np.isfinite(m)                                   # rows that see at least one key
        e = np.exp(s[rows] - m[rows, None])
        den = e.sum(axis=1)
        lse[a, rows] = m[rows] + np.log(den)
        o[rows, a] = (e / den[:, None]) @ v[:, g]
    return o, lse


def merge(o_a, lse_a, o_b, lse_b):
    """O [S,H,D], LSE [H,S] of two disjoint key sets -> those of their union."""
    o_a = np.asarray(o_a, np.float64); o_b = np.asarray(o_b, np.float64)
    lse_a = np.asarray(lse_a, np.float64); lse_b = np.asarray(lse_b, np.float64)
    lse = np.logaddexp(lse_a, lse_b)
    with np.errstate(invalid="ignore"):
        wa = np.where(np.isfinite(lse), np.exp(lse_a - lse), 0.0)   # [H,S]
        wb = np.where(np.isfinite(lse), np.exp(lse_b - lse), 0.0)
    o = wa.T[:, :, None] * o_a + wb.T[:, :, None] * o_b
    return o, lse


def block_attn_bwd(q, k, v, lse, delta, do, scale: float, off: int):
    """Shares of dQ [Sq,Hq,D], dK, dV [Skv,Hkv,D] from this block pair.
    lse, delta: [Hq,Sq], of the final output."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    do = np.asarray(do, np.float64)
    lse = np.asarray(lse, np.float64); delta = np.asarray(delta, np.float64)
    Sq, Hq, D = q.shape
    Skv, Hkv, _ = k.shape
    G = Hq // Hkv
    vis = _visible(Sq, Skv, off)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    for a in range(Hq):
        g = a // G
        with np.errstate(invalid="ignore"):
            p = np.where(vis, np.exp(scale * (q[:, a] @ k[:, g].T) - lse[a][:, None]), 0.0)
        dp = do[:, a] @ v[:, g].T
        ds = p * (dp - delta[a][:, None])
        dq[:, a] = scale * (ds @ k[:, g])
        dk[:, g] += scale * (ds.T @ q[:, a])
        dv[:, g] += p.T @ do[:, a]
    return dq, dk, dv
