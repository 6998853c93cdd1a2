"""Attention on sequence-side tensors (the re-layout folded into the attention
kernels' loads and stores): bit-identical to pack -> attention -> unpack, and
within the parity bars of the fp64 oracle run on the oracle's own re-layout."""
import numpy as np
import pytest
import torch

from oracle import ref_numpy as rn
from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import synth
from gpu_util import GRAD_REL_L2, LSE_MAX_ABS, check_o, dev_bf16, host_f64, grad_err

pytestmark = pytest.mark.gpu


def seq_side_inputs(seed, B, S_l, Hq, Hkv, D, P):
    """Sequence-side bf16 bit tensors: [B, S_l, P*H, D]."""
    q, k, v, do = synth.attn_inputs(seed, S_l, P * Hq, P * Hkv, D, B)
    return q, k, v, do


def bits(t):
    return t.contiguous().view(torch.int16)


CASES = [
    # B, S_l, Hq, Hkv, D, P
    (1, 256, 2, 1, 64, 4),     # tiny-config head counts: one WG tile per chunk
    (1, 512, 4, 1, 128, 2),
    (2, 256, 2, 2, 128, 3),    # batch, three chunks (P need not be a power of two)
    (1, 1024, 4, 1, 128, 8),   # 8192 attention rows: dK/dV key tiles shared by several workgroups
]


@pytest.mark.parametrize("B,S_l,Hq,Hkv,D,P", CASES)
def test_seqlayout_equals_pack_attention_unpack_bitwise(B, S_l, Hq, Hkv, D, P):
    q, k, v, do = (dev_bf16(t) for t in seq_side_inputs(S_l + P, B, S_l, Hq, Hkv, D, P))
    # reference path: the three steps the folded kernels replace
    qa, ka, va, doa = (sp.sp_pack_seq_to_head(t, P) for t in (q, k, v, do))
    oa, lse_a = sp.sp_attn_fwd(qa, ka, va)
    dqa, dka, dva = sp.sp_attn_bwd(qa, ka, va, oa, lse_a, doa)
    want = [sp.sp_unpack_head_to_seq(t, P) for t in (oa, dqa, dka, dva)]
    # folded path
    o, lse = sp.sp_attn_fwd_seqlayout(q, k, v, P)
    dq, dk, dv = sp.sp_attn_bwd_seqlayout(q, k, v, o, lse, do, P)
    torch.cuda.synchronize()
    assert torch.equal(lse, lse_a)
    for name, got, ref in zip(("O", "dQ", "dK", "dV"), (o, dq, dk, dv), want):
        assert torch.equal(bits(got), bits(ref)), name


def test_seqlayout_matches_oracle():
    B, S_l, Hq, Hkv, D, P = 1, 256, 2, 1, 128, 4
    q, k, v, do = seq_side_inputs(5, B, S_l, Hq, Hkv, D, P)
    qd, kd, vd, dod = (dev_bf16(t) for t in (q, k, v, do))
    o, lse = sp.sp_attn_fwd_seqlayout(qd, kd, vd, P)
    dq, dk, dv = sp.sp_attn_bwd_seqlayout(qd, kd, vd, o, lse, dod, P)
    torch.cuda.synchronize()
    # oracle: its own pack, dense attention, its own unpack
    qa, ka, va, doa = (rn.pack_seq_to_head(rn.widen_bf16(t[0]), P) for t in (q, k, v, do))
    o_r, lse_r = rn.attn_fwd(qa, ka, va)
    dq_r, dk_r, dv_r, _ = rn.attn_bwd(qa, ka, va, doa)
    un = lambda x: rn.unpack_head_to_seq(x, P)
    check_o(host_f64(o)[0], un(o_r), "seq-layout O")
    assert np.abs(host_f64(lse)[0] - lse_r).max() <= LSE_MAX_ABS
    e = (grad_err(host_f64(dq)[0], un(dq_r)), grad_err(host_f64(dk)[0], un(dk_r)), grad_err(host_f64(dv)[0], un(dv_r)))
    print(f"seq-layout: rel-L2 dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert max(e) <= GRAD_REL_L2


def test_seqlayout_full_size_shard_bitwise():
    """The 8B-shaped shard at 32K rows (S_l = 4096, P = 8), forward and backward."""
    cfg = synth.CONFIGS["c2_8b_32k"]
    S_l, P, Hq, Hkv, D = cfg["pack"]["S_l"], cfg["pack"]["P"], cfg["Hq"], cfg["Hkv"], cfg["D"]
    g = torch.Generator(device="cuda").manual_seed(3)
    mk = lambda h: torch.randn((1, S_l, P * h, D), device="cuda", generator=g).to(torch.bfloat16)
    q, k, v, do = mk(Hq), mk(Hkv), mk(Hkv), mk(Hq)
    qa, ka, va, doa = (sp.sp_pack_seq_to_head(t, P) for t in (q, k, v, do))
    oa, lse_a = sp.sp_attn_fwd(qa, ka, va)
    dqa, dka, dva = sp.sp_attn_bwd(qa, ka, va, oa, lse_a, doa)
    want = [sp.sp_unpack_head_to_seq(t, P) for t in (oa, dqa, dka, dva)]
    o, lse = sp.sp_attn_fwd_seqlayout(q, k, v, P)
    dq, dk, dv = sp.sp_attn_bwd_seqlayout(q, k, v, o, lse, do, P)
    torch.cuda.synchronize()
    assert torch.equal(lse, lse_a)
    for name, got, ref in zip(("O", "dQ", "dK", "dV"), (o, dq, dk, dv), want):
        assert torch.equal(bits(got), bits(ref)), name
