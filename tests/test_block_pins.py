"""Pins for the blockwise-attention oracle (oracle/ref_block.py): scalar brute
force, a library softmax, the special cases that reduce to functions pinned
elsewhere, the union-of-key-sets identity of the merge, and sums of per-block
gradient shares against torch fp64 autograd of attention over the whole
sequence.  CPU only."""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import ref_block as rb
from oracle import ref_numpy as rn


def rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def brute_fwd(q, k, v, scale, off):
    """One (row, head) at a time with Python scalars."""
    Sq, Hq, D = q.shape
    Skv, Hkv, _ = k.shape
    G = Hq // Hkv
    o = np.zeros((Sq, Hq, D)); lse = np.full((Hq, Sq), -np.inf)
    for i in range(Sq):
        for a in range(Hq):
            g = a // G
            js = [j for j in range(Skv) if j <= i + off]
            if not js:
                continue
            s = [scale * sum(q[i, a, d] * k[j, g, d] for d in range(D)) for j in js]
            m = max(s)
            den = sum(math.exp(x - m) for x in s)
            lse[a, i] = m + math.log(den)
            for x, j in zip(s, js):
                o[i, a] += math.exp(x - m) / den * v[j, g]
    return o, lse


@pytest.mark.parametrize("Sq,Skv,Hq,Hkv,off", [(5, 7, 2, 1, 0), (6, 4, 4, 2, 2), (4, 9, 1, 1, 20), (7, 5, 2, 2, -3)])
def test_block_fwd_brute_force(Sq, Skv, Hq, Hkv, off):
    q, k, v = rand(1, Sq, Hq, 4), rand(2, Skv, Hkv, 4), rand(3, Skv, Hkv, 4)
    o, lse = rb.block_attn_fwd(q, k, v, 0.37, off)
    o_b, lse_b = brute_fwd(q, k, v, 0.37, off)
    np.testing.assert_allclose(o, o_b, rtol=1e-12, atol=1e-14)
    np.testing.assert_array_equal(np.isinf(lse), np.isinf(lse_b))
    f = np.isfinite(lse_b)
    np.testing.assert_allclose(lse[f], lse_b[f], rtol=1e-12)


def test_block_fwd_unmasked_is_library_softmax():
    Sq, Skv, H, D = 9, 13, 2, 8
    q, k, v = rand(4, Sq, H, D), rand(5, Skv, H, D), rand(6, Skv, H, D)
    scale = 0.2
    o, lse = rb.block_attn_fwd(q, k, v, scale, Skv - 1)
    for a in range(H):
        s = scale * q[:, a] @ k[:, a].T
        np.testing.assert_allclose(o[:, a], scipy.special.softmax(s, axis=1) @ v[:, a], rtol=1e-12)
        np.testing.assert_allclose(lse[a], scipy.special.logsumexp(s, axis=1), rtol=1e-12)


def test_block_fwd_diagonal_block_is_causal_attention():
    S, Hq, Hkv, D = 33, 4, 2, 8
    q, k, v = rand(7, S, Hq, D), rand(8, S, Hkv, D), rand(9, S, Hkv, D)
    o, lse = rb.block_attn_fwd(q, k, v, 0.3, 0)
    o_c, lse_c = rn.attn_fwd(q, k, v, 0.3)
    np.testing.assert_allclose(o, o_c, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, lse_c, rtol=1e-12)


def test_merge_is_softmax_over_the_union():
    Sq, H, D = 6, 2, 4
    q = rand(10, Sq, H, D)
    k, v = rand(11, 11, H, D), rand(12, 11, H, D)
    scale = 0.5
    full = rb.block_attn_fwd(q, k, v, scale, 100)
    a = rb.block_attn_fwd(q, k[:4], v[:4], scale, 100)
    b = rb.block_attn_fwd(q, k[4:], v[4:], scale, 100)
    o, lse = rb.merge(*a, *b)
    np.testing.assert_allclose(o, full[0], rtol=1e-12)
    np.testing.assert_allclose(lse, full[1], rtol=1e-12)
    # order does not matter; an empty set is the identity
    o2, lse2 = rb.merge(*b, *a)
    np.testing.assert_allclose(o2, o, rtol=1e-14)
    np.testing.assert_allclose(lse2, lse, rtol=1e-14)
    o3, lse3 = rb.merge(np.zeros_like(o), np.full_like(lse, -np.inf), *a)
    np.testing.assert_array_equal(o3, a[0])
    np.testing.assert_array_equal(lse3, a[1])
    o4, lse4 = rb.merge(np.zeros_like(o), np.full_like(lse, -np.inf), np.zeros_like(o), np.full_like(lse, -np.inf))
    assert np.all(o4 == 0) and np.all(np.isneginf(lse4))


def ring(q, k, v, scale, bounds_q, bounds_k):
    """Forward of every query block against every key block that it can see, merged."""
    S, Hq, D = q.shape
    o = np.zeros((S, Hq, D)); lse = np.full((Hq, S), -np.inf)
    for a0, a1 in bounds_q:
        acc = (np.zeros((a1 - a0, Hq, D)), np.full((Hq, a1 - a0), -np.inf))
        for c0, c1 in bounds_k:
            blk = rb.block_attn_fwd(q[a0:a1], k[c0:c1], v[c0:c1], scale, a0 - c0)
            acc = rb.merge(*acc, *blk)
        o[a0:a1], lse[:, a0:a1] = acc
    return o, lse


@pytest.mark.parametrize("bq,bk", [([0, 8, 16, 24], [0, 8, 16, 24]), ([0, 5, 24], [0, 3, 11, 24]), ([0, 24], [0, 7, 24])])
def test_ring_of_blocks_is_causal_attention(bq, bk):
    S, Hq, Hkv, D = 24, 4, 2, 8
    q, k, v = rand(13, S, Hq, D), rand(14, S, Hkv, D), rand(15, S, Hkv, D)
    o, lse = ring(q, k, v, 0.25, list(zip(bq[:-1], bq[1:])), list(zip(bk[:-1], bk[1:])))
    o_c, lse_c = rn.attn_fwd(q, k, v, 0.25)
    np.testing.assert_allclose(o, o_c, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(lse, lse_c, rtol=1e-11)


def torch_causal(q, k, v, scale):
    S, Hq, D = q.shape
    G = Hq // k.shape[1]
    kk = k.repeat_interleave(G, dim=1); vv = v.repeat_interleave(G, dim=1)
    s = scale * torch.einsum("ihd,jhd->hij", q, kk)
    s = s.masked_fill(~torch.tril(torch.ones(S, S, dtype=torch.bool)), float("-inf"))
    return torch.einsum("hij,jhd->ihd", torch.softmax(s, dim=-1), vv)


@pytest.mark.parametrize("bq,bk", [([0, 8, 16, 24], [0, 8, 16, 24]), ([0, 5, 24], [0, 3, 11, 24])])
def test_block_bwd_shares_sum_to_autograd(bq, bk):
    S, Hq, Hkv, D = 24, 4, 2, 8
    scale = 0.25
    q, k, v, do = rand(16, S, Hq, D), rand(17, S, Hkv, D), rand(18, S, Hkv, D), rand(19, S, Hq, D)
    tq, tk, tv = (torch.tensor(t, dtype=torch.float64, requires_grad=True) for t in (q, k, v))
    out = torch_causal(tq, tk, tv, scale)
    (out * torch.tensor(do)).sum().backward()
    o, lse = rn.attn_fwd(q, k, v, scale)
    np.testing.assert_allclose(o, out.detach().numpy(), rtol=1e-11, atol=1e-13)
    delta = np.einsum("shd,shd->hs", o, do)
    dq = np.zeros_like(q); dk = np.zeros_like(k); dv = np.zeros_like(v)
    for a0, a1 in zip(bq[:-1], bq[1:]):
        for c0, c1 in zip(bk[:-1], bk[1:]):
            if c0 > a1 - 1:
                continue  # nothing visible
            sq, sk, sv = rb.block_attn_bwd(q[a0:a1], k[c0:c1], v[c0:c1], lse[:, a0:a1], delta[:, a0:a1],
                                           do[a0:a1], scale, a0 - c0)
            dq[a0:a1] += sq; dk[c0:c1] += sk; dv[c0:c1] += sv
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_block_bwd_single_block_is_causal_backward():
    S, Hq, Hkv, D = 19, 2, 1, 8
    q, k, v, do = rand(20, S, Hq, D), rand(21, S, Hkv, D), rand(22, S, Hkv, D), rand(23, S, Hq, D)
    dq_c, dk_c, dv_c, delta = rn.attn_bwd(q, k, v, do, 0.4)
    _, lse = rn.attn_fwd(q, k, v, 0.4)
    dq, dk, dv = rb.block_attn_bwd(q, k, v, lse, delta, do, 0.4, 0)
    np.testing.assert_allclose(dq, dq_c, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dk, dk_c, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dv, dv_c, rtol=1e-11, atol=1e-13)
