"""Parity of the HIP attention forward with the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import ref_numpy as rn
from oracle import ref_stream as rs
from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import synth
from gpu_util import LSE_MAX_ABS, check_o, dev_bf16, host_f64

pytestmark = pytest.mark.gpu

SMALL = [
    # S, Hq, Hkv, D, B
    (512, 2, 1, 64, 1),    # tiny config
    (1, 1, 1, 64, 1),
    (31, 2, 2, 128, 1),
    (64, 4, 1, 128, 2),
    (129, 3, 1, 64, 1),    # one row past a 128-row tile
    (200, 8, 2, 128, 1),
    (1000, 4, 1, 128, 1),  # several tiles and a ragged tail
    (777, 2, 2, 64, 3),
    (600, 3, 1, 128, 1),   # Llama-3.2 3B-shaped shard: 3 query heads on one KV head
    (520, 5, 5, 128, 1),   # Llama-2 13B-shaped shard: full attention, 5 heads
]


@pytest.mark.parametrize("S,Hq,Hkv,D,B", SMALL)
def test_fwd_matches_oracle(S, Hq, Hkv, D, B):
    q, k, v, _ = synth.attn_inputs(S + D, S, Hq, Hkv, D, B)
    o, lse = sp.sp_attn_fwd(dev_bf16(q), dev_bf16(k), dev_bf16(v))
    torch.cuda.synchronize()
    og, lg = host_f64(o), host_f64(lse)
    for b in range(B):
        o_ref, l_ref = rn.attn_fwd(rn.widen_bf16(q[b]), rn.widen_bf16(k[b]), rn.widen_bf16(v[b]))
        err = check_o(og[b], o_ref, f"S={S}")
        lerr = np.abs(lg[b] - l_ref).max()
        assert lerr <= LSE_MAX_ABS, f"LSE max-abs {lerr:.3e}"
        print(f"S={S} Hq={Hq} Hkv={Hkv} D={D} b={b}: O max-abs {err:.2e}, LSE max-abs {lerr:.2e}")


def test_fwd_explicit_scale_and_determinism():
    S, Hq, Hkv, D = 300, 4, 2, 128
    q, k, v, _ = synth.attn_inputs(3, S, Hq, Hkv, D)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    o1, l1 = sp.sp_attn_fwd(qd, kd, vd, softmax_scale=0.2)
    o2, l2 = sp.sp_attn_fwd(qd, kd, vd, softmax_scale=0.2)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16)) and torch.equal(l1, l2)
    o_ref, l_ref = rn.attn_fwd(rn.widen_bf16(q[0]), rn.widen_bf16(k[0]), rn.widen_bf16(v[0]), 0.2)
    check_o(host_f64(o1)[0], o_ref)
    assert np.abs(host_f64(l1)[0] - l_ref).max() <= LSE_MAX_ABS


def test_fwd_closed_forms_on_device():
    """Zero queries give prefix means of V and LSE = ln(i+1); constant V gives
    constant O: no oracle involved."""
    S, Hq, Hkv, D = 260, 2, 1, 128
    _, k, v, _ = synth.attn_inputs(4, S, Hq, Hkv, D)
    kd, vd = dev_bf16(k), dev_bf16(v)
    qd = torch.zeros((1, S, Hq, D), dtype=torch.bfloat16, device="cuda")
    o, lse = sp.sp_attn_fwd(qd, kd, vd)
    vf = synth.bf16_bits_to_f32(v)[0].astype(np.float64)
    pm = np.cumsum(vf, axis=0) / np.arange(1, S + 1)[:, None, None]
    assert np.abs(host_f64(o)[0] - np.repeat(pm, Hq, axis=1)).max() <= 1e-2
    assert np.abs(host_f64(lse)[0] - np.log(np.arange(1, S + 1))).max() <= 1e-5
    q, _, _, _ = synth.attn_inputs(5, S, Hq, Hkv, D)
    ones = torch.full((1, S, Hkv, D), 1.25, dtype=torch.bfloat16, device="cuda")
    o2, _ = sp.sp_attn_fwd(dev_bf16(q), kd, ones)
    assert np.abs(host_f64(o2) - 1.25).max() <= 2 ** -7


@pytest.mark.parametrize("name", ["c2_8b_32k", "c3_8b_128k", "c4_70b_128k"])
def test_fwd_full_size_sampled_rows(name):
    """Full-size shards in the launch configuration the benchmark times; the
    oracle computes sampled rows one by one: tile edges, the first and last
    rows, and random rows."""
    cfg = synth.CONFIGS[name]
    S, Hq, Hkv, D = cfg["S"], cfg["Hq"], cfg["Hkv"], cfg["D"]
    q, k, v, _ = synth.attn_inputs(0, S, Hq, Hkv, D)
    o, lse = sp.sp_attn_fwd(dev_bf16(q), dev_bf16(k), dev_bf16(v))
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    rows = np.unique(np.concatenate([
        [0, 1, 31, 32, 63, 64, 127, 128, 129, S // 2 - 1, S // 2, S - 129, S - 128, S - 65, S - 64, S - 1],
        rng.integers(0, S, 48)]))
    r = rs.attn_rows(rn.widen_bf16(q[0]), rn.widen_bf16(k[0]), rn.widen_bf16(v[0]), rows)
    og = host_f64(o[0, torch.from_numpy(rows).cuda()])
    lg = host_f64(lse[0][:, torch.from_numpy(rows).cuda()])
    err = check_o(og, r["O"], name)
    lerr = np.abs(lg - r["lse"]).max()
    print(f"{name}: sampled {rows.size} rows, O max-abs {err:.2e}, LSE max-abs {lerr:.2e}")
    assert lerr <= LSE_MAX_ABS
    # any-size properties: LSE_i >= s_ii (the diagonal term is part of the sum)
    qf = synth.bf16_bits_to_f32(q[0]).astype(np.float64)
    kf = synth.bf16_bits_to_f32(k[0]).astype(np.float64)
    sii = np.einsum("iad,iad->ai", qf, np.repeat(kf, Hq // Hkv, axis=1)) / np.sqrt(D)
    assert np.all(host_f64(lse)[0] >= sii - 1e-3)
    assert torch.isfinite(o.float()).all()
