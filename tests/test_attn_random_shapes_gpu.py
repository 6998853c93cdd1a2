"""Seeded random extents (rows, keys, heads, group size, head dim, batch, causal
offset, packed documents) through every attention entry point, each compared
element by element with the fp64 oracle.  Sizes stay small enough for the dense
oracle and still cover several tiles, ragged tails and single-row corners."""
import numpy as np
import pytest
import torch

from oracle import ref_block as rb
from oracle import ref_numpy as rn
from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import synth
from gpu_util import GRAD_REL_L2, LSE_MAX_ABS, check_o, dev_bf16, host_f64, grad_err

pytestmark = pytest.mark.gpu


def draw_heads(rng):
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 3, 4, 8]))
    return Hkv * G, Hkv


def draw_len(rng):
    """Mostly a few tiles, sometimes a corner (1 row, one short of / exactly / one past a tile edge)."""
    if rng.random() < 0.3:
        return int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, 255, 256, 257, 511, 512, 513]))
    return int(rng.integers(1, 900))


@pytest.mark.parametrize("seed", range(12))
def test_random_causal_fwd_bwd(seed):
    rng = np.random.default_rng(1000 + seed)
    S, (Hq, Hkv), D, B = draw_len(rng), draw_heads(rng), int(rng.choice([64, 128])), int(rng.choice([1, 1, 2]))
    scale = float(rng.choice([0.0, 0.05, 0.2]))
    qb, kb, vb, dob = synth.attn_inputs(seed, S, Hq, Hkv, D, B)
    q, k, v, do = (dev_bf16(t) for t in (qb, kb, vb, dob))
    o, lse = sp.sp_attn_fwd(q, k, v, softmax_scale=scale)
    dq, dk, dv = sp.sp_attn_bwd(q, k, v, o, lse, do, softmax_scale=scale)
    torch.cuda.synchronize()
    for b in range(B):
        f = [rn.widen_bf16(t[b]) for t in (qb, kb, vb, dob)]
        o_ref, lse_ref = rn.attn_fwd(f[0], f[1], f[2], scale)
        check_o(host_f64(o)[b], o_ref, f"S={S} Hq={Hq} Hkv={Hkv} D={D} b={b}")
        assert np.abs(host_f64(lse)[b] - lse_ref).max() <= LSE_MAX_ABS
        rq, rk, rv, _ = rn.attn_bwd(*f, scale)
        for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
            err = grad_err(host_f64(got)[b], ref)
            assert err <= GRAD_REL_L2, f"{name} S={S} Hq={Hq} Hkv={Hkv} D={D} b={b}: rel L2 {err:.3e}"


@pytest.mark.parametrize("seed", range(16))
def test_random_block_fwd_bwd(seed):
    rng = np.random.default_rng(2000 + seed)
    Sq, Skv, (Hq, Hkv), D = draw_len(rng), draw_len(rng), draw_heads(rng), int(rng.choice([64, 128]))
    lo = max(0, Skv - Sq)                       # every key must be seen by some row
    off = int(rng.choice([lo, lo + int(rng.integers(0, 300)), Skv - 1 if Skv - 1 >= lo else lo, Skv + 5]))
    scale = 1.0 / np.sqrt(D)
    qb, _, _, dob = synth.attn_inputs(seed, Sq, Hq, Hkv, D)
    _, kb, vb, _ = synth.attn_inputs(seed + 500, Skv, Hq, Hkv, D)
    q, k, v, do = (dev_bf16(t) for t in (qb, kb, vb, dob))
    o, lse = sp.sp_attn_block_fwd(q, k, v, off)
    dq, dk, dv = sp.sp_attn_block_bwd(q, k, v, o, lse, do, off)
    torch.cuda.synchronize()
    q64, k64, v64, do64 = (rn.widen_bf16(t[0]) for t in (qb, kb, vb, dob))
    what = f"Sq={Sq} Skv={Skv} Hq={Hq} Hkv={Hkv} D={D} off={off}"
    o_ref, lse_ref = rb.block_attn_fwd(q64, k64, v64, scale, off)
    check_o(host_f64(o)[0], o_ref, what)
    assert np.abs(host_f64(lse)[0] - lse_ref).max() <= LSE_MAX_ABS, what
    delta_ref = np.einsum("shd,shd->hs", o_ref, do64)
    rq, rk, rv = rb.block_attn_bwd(q64, k64, v64, lse_ref, delta_ref, do64, scale, off)
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        err = grad_err(host_f64(got)[0], ref)
        assert err <= GRAD_REL_L2, f"{name} {what}: rel L2 {err:.3e}"


@pytest.mark.parametrize("seed", range(8))
def test_random_packed_documents(seed):
    rng = np.random.default_rng(3000 + seed)
    n_docs = int(rng.integers(1, 9))
    lengths = [int(draw_len(rng) if rng.random() < 0.8 else 0) for _ in range(n_docs)]
    if sum(lengths) == 0:
        lengths[0] = 17
    T, (Hq, Hkv), D = sum(lengths), draw_heads(rng), int(rng.choice([64, 128]))
    cu_h = synth.cu_seqlens_from_lengths(lengths)
    cu = torch.from_numpy(cu_h).cuda()
    qb, kb, vb, dob = synth.attn_inputs(seed, T, Hq, Hkv, D)
    q, k, v, do = (dev_bf16(t[0]) for t in (qb, kb, vb, dob))
    o, lse = sp.sp_attn_varlen_fwd(q, k, v, cu)
    dq, dk, dv = sp.sp_attn_varlen_bwd(q, k, v, o, lse, do, cu)
    torch.cuda.synchronize()
    f = [rn.widen_bf16(t[0]) for t in (qb, kb, vb, dob)]
    what = f"lengths={lengths} Hq={Hq} Hkv={Hkv} D={D}"
    o_ref, lse_ref = rn.attn_varlen_fwd(f[0], f[1], f[2], cu_h)
    check_o(host_f64(o), o_ref, what)
    assert np.abs(host_f64(lse) - lse_ref).max() <= LSE_MAX_ABS, what
    rq, rk, rv, _ = rn.attn_varlen_bwd(*f, cu_h)
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        err = grad_err(host_f64(got), ref)
        assert err <= GRAD_REL_L2, f"{name} {what}: rel L2 {err:.3e}"
