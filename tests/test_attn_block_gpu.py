"""Blockwise attention step of a ring schedule on the GPU (block forward, merge,
per-block gradient shares) against the fp64 oracle, element by element, and the
cases that must reproduce the plain causal entry points bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ref_block as rb
from oracle import ref_numpy as rn
from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import synth
from gpu_util import GRAD_REL_L2, LSE_MAX_ABS, check_o, dev_bf16, host_f64, grad_err

pytestmark = pytest.mark.gpu


def block_inputs(seed, Sq, Skv, Hq, Hkv, D, B=1):
    """Seeded bf16 bit tensors of a query block and a key/value block."""
    q, _, _, do = synth.attn_inputs(seed, Sq, Hq, Hkv, D, B)
    _, k, v, _ = synth.attn_inputs(seed + 1000, Skv, Hq, Hkv, D, B)
    return q, k, v, do


def bits(t):
    return t.contiguous().view(torch.int16)


FWD_CASES = [
    # Sq, Skv, Hq, Hkv, D, causal_offset
    (300, 300, 4, 2, 128, 0),      # the diagonal block, ragged
    (300, 520, 4, 2, 128, 520),    # a block from the past: nothing hidden, ragged on both sides
    (256, 256, 2, 1, 64, 255),     # smallest offset that hides nothing
    (200, 333, 3, 1, 128, 140),    # a diagonal that crosses the block
    (520, 100, 5, 5, 128, 0),      # fewer keys than rows
    (1, 700, 2, 2, 64, 699),       # a single query row
    (777, 64, 4, 1, 128, 5),       # one key tile
]


@pytest.mark.parametrize("Sq,Skv,Hq,Hkv,D,off", FWD_CASES)
def test_block_fwd_matches_oracle(Sq, Skv, Hq, Hkv, D, off):
    q, k, v, _ = block_inputs(Sq + Skv, Sq, Skv, Hq, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    o, lse = sp.sp_attn_block_fwd(dev_bf16(q), dev_bf16(k), dev_bf16(v), off)
    torch.cuda.synchronize()
    o_ref, lse_ref = rb.block_attn_fwd(rn.widen_bf16(q[0]), rn.widen_bf16(k[0]), rn.widen_bf16(v[0]), scale, off)
    check_o(host_f64(o)[0], o_ref, "block fwd")
    assert np.abs(host_f64(lse)[0] - lse_ref).max() <= LSE_MAX_ABS


def test_block_fwd_batched():
    B, Sq, Skv, Hq, Hkv, D, off = 2, 260, 400, 4, 1, 128, 150
    q, k, v, _ = block_inputs(5, Sq, Skv, Hq, Hkv, D, B)
    o, lse = sp.sp_attn_block_fwd(dev_bf16(q), dev_bf16(k), dev_bf16(v), off, softmax_scale=0.11)
    torch.cuda.synchronize()
    for b in range(B):
        o_ref, lse_ref = rb.block_attn_fwd(rn.widen_bf16(q[b]), rn.widen_bf16(k[b]), rn.widen_bf16(v[b]), 0.11, off)
        check_o(host_f64(o)[b], o_ref, f"block fwd batch {b}")
        assert np.abs(host_f64(lse)[b] - lse_ref).max() <= LSE_MAX_ABS


@pytest.mark.parametrize("S,Hq,Hkv,D", [(520, 4, 2, 128), (2304, 4, 1, 128), (300, 2, 2, 64)])
def test_diagonal_block_is_the_causal_entry_point_bitwise(S, Hq, Hkv, D):
    q, k, v, do = (dev_bf16(t) for t in synth.attn_inputs(S, S, Hq, Hkv, D))
    o, lse = sp.sp_attn_fwd(q, k, v)
    ob, lseb = sp.sp_attn_block_fwd(q, k, v, 0)
    assert torch.equal(bits(o), bits(ob)) and torch.equal(lse, lseb)
    g = sp.sp_attn_bwd(q, k, v, o, lse, do)
    gb = sp.sp_attn_block_bwd(q, k, v, o, lse, do, 0)
    torch.cuda.synchronize()
    for x, y in zip(g, gb):
        assert torch.equal(bits(x), bits(y))


def test_merge_matches_oracle():
    B, S, Hq, D = 2, 333, 3, 128
    rng = np.random.default_rng(7)
    o_acc = rng.standard_normal((B, S, Hq, D)).astype(np.float32)
    o_blk = synth.normal_bf16(rng, (B, S, Hq, D))
    lse_acc = (3.0 * rng.standard_normal((B, Hq, S))).astype(np.float32)
    lse_blk = (3.0 * rng.standard_normal((B, Hq, S))).astype(np.float32)
    # rows that have seen no key yet, rows whose block is empty, and both
    lse_acc[:, :, 0:40] = -np.inf
    o_acc[:, 0:40] = 0.0
    lse_blk[:, :, 20:60] = -np.inf
    o_blk[:, 20:60] = 0
    d_acc, d_lse = torch.from_numpy(o_acc).cuda(), torch.from_numpy(lse_acc).cuda()
    o_out = torch.empty((B, S, Hq, D), dtype=torch.bfloat16, device="cuda")
    sp.sp_attn_merge(d_acc, d_lse, dev_bf16(o_blk), torch.from_numpy(lse_blk).cuda(), o_out)
    torch.cuda.synchronize()
    for b in range(B):
        o_ref, lse_ref = rb.merge(o_acc[b], lse_acc[b], rn.widen_bf16(o_blk[b]), lse_blk[b])
        got_lse = host_f64(d_lse)[b]
        empty = np.isneginf(lse_ref)
        assert empty[:, 20:40].all() and np.array_equal(np.isneginf(got_lse), empty)
        assert np.abs(got_lse[~empty] - lse_ref[~empty]).max() <= 1e-5
        # fp32 arithmetic on O(1) values
        assert np.abs(host_f64(d_acc)[b] - o_ref).max() <= 1e-5
        # the bf16 copy is the rounding of the fp32 result
        assert torch.equal(bits(o_out[b]), bits(d_acc[b].to(torch.bfloat16)))


def ring_forward(q, k, v, n, scale=0.0):
    """Every query block against every key block it can see, merged on the device.  Returns bf16 O, fp32 LSE."""
    B, S, Hq, D = q.shape
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, S), dtype=torch.float32, device="cuda")
    for a0 in range(0, S, n):
        a1 = min(a0 + n, S)
        o_acc = torch.zeros((B, a1 - a0, Hq, D), dtype=torch.float32, device="cuda")
        lse_acc = torch.full((B, Hq, a1 - a0), -np.inf, dtype=torch.float32, device="cuda")
        o_fin = torch.empty((B, a1 - a0, Hq, D), dtype=torch.bfloat16, device="cuda")
        for c0 in range(0, a1, n):
            c1 = min(c0 + n, S)
            ob, lb = sp.sp_attn_block_fwd(q[:, a0:a1].contiguous(), k[:, c0:c1].contiguous(),
                                          v[:, c0:c1].contiguous(), a0 - c0, softmax_scale=scale)
            sp.sp_attn_merge(o_acc, lse_acc, ob, lb, o_fin if c0 + n >= a1 else None)
        o[:, a0:a1] = o_fin
        lse[:, :, a0:a1] = lse_acc
    return o, lse


RING_CASES = [
    # S, block, Hq, Hkv, D
    (1536, 512, 4, 2, 128),
    (1300, 400, 2, 1, 64),     # ragged blocks, last one short
    (4096, 1024, 4, 1, 128),   # dK/dV key tiles shared by several workgroups
]


@pytest.mark.parametrize("S,n,Hq,Hkv,D", RING_CASES)
def test_ring_of_blocks_matches_oracle(S, n, Hq, Hkv, D):
    """Forward and backward of causal attention computed block by block, as a ring schedule would on one
    device after the other: the merged forward and every block pair's gradient shares against the oracle."""
    qb, kb, vb, dob = synth.attn_inputs(S + n, S, Hq, Hkv, D)
    q, k, v, do = (dev_bf16(t) for t in (qb, kb, vb, dob))
    scale = 1.0 / np.sqrt(D)
    o, lse = ring_forward(q, k, v, n)
    torch.cuda.synchronize()
    q64, k64, v64, do64 = (rn.widen_bf16(t[0]) for t in (qb, kb, vb, dob))
    o_ref, lse_ref = rn.attn_fwd(q64, k64, v64)
    check_o(host_f64(o)[0], o_ref, "ring fwd")
    assert np.abs(host_f64(lse)[0] - lse_ref).max() <= LSE_MAX_ABS

    delta_ref = np.einsum("shd,shd->hs", o_ref, do64)
    dq_sum = np.zeros_like(q64); dk_sum = np.zeros_like(k64); dv_sum = np.zeros_like(v64)
    for a0 in range(0, S, n):
        a1 = min(a0 + n, S)
        qa, oa, doa = (t[:, a0:a1].contiguous() for t in (q, o, do))
        la = lse[:, :, a0:a1].contiguous()
        ws = None
        for c0 in range(0, a1, n):
            c1 = min(c0 + n, S)
            kc, vc = k[:, c0:c1].contiguous(), v[:, c0:c1].contiguous()
            if ws is None:
                need = max(sp.sp_attn_block_bwd_workspace_bytes(1, a1 - a0, min(x + n, S) - x, Hq, Hkv, D)
                           for x in range(0, a1, n))
                ws = torch.empty(need, dtype=torch.uint8, device="cuda")
                stages = sp.SP_BWD_STAGE_ALL
            else:
                stages = sp.SP_BWD_STAGE_DKDV | sp.SP_BWD_STAGE_DQ  # Delta of these rows is in the workspace
            dq, dk, dv = sp.sp_attn_block_bwd(qa, kc, vc, oa, la, doa, a0 - c0, workspace=ws, stages=stages)
            torch.cuda.synchronize()
            rq, rk, rv = rb.block_attn_bwd(q64[a0:a1], k64[c0:c1], v64[c0:c1], lse_ref[:, a0:a1],
                                           delta_ref[:, a0:a1], do64[a0:a1], scale, a0 - c0)
            for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
                err = grad_err(host_f64(got)[0], ref)
                assert err <= GRAD_REL_L2, f"{name} share of rows {a0}.. keys {c0}..: rel L2 {err:.3e}"
            dq_sum[a0:a1] += host_f64(dq)[0]; dk_sum[c0:c1] += host_f64(dk)[0]; dv_sum[c0:c1] += host_f64(dv)[0]
    fq, fk, fv, _ = rn.attn_bwd(q64, k64, v64, do64)
    for name, got, ref in (("dq", dq_sum, fq), ("dk", dk_sum, fk), ("dv", dv_sum, fv)):
        err = grad_err(got, ref)
        assert err <= GRAD_REL_L2, f"{name} summed over blocks: rel L2 {err:.3e}"


BWD_CASES = [
    # Sq, Skv, Hq, Hkv, D, causal_offset: rectangular pairs a ring never produces with equal blocks
    (200, 333, 3, 1, 128, 140),
    (520, 100, 5, 5, 128, 0),
    (64, 2100, 4, 2, 64, 2099),
    (2100, 300, 4, 1, 128, 7),
]


@pytest.mark.parametrize("Sq,Skv,Hq,Hkv,D,off", BWD_CASES)
def test_block_bwd_rectangular_matches_oracle(Sq, Skv, Hq, Hkv, D, off):
    """A lone block pair: its own forward gives the final O and LSE."""
    qb, kb, vb, dob = block_inputs(Sq * 3 + Skv, Sq, Skv, Hq, Hkv, D)
    q, k, v, do = (dev_bf16(t) for t in (qb, kb, vb, dob))
    scale = 1.0 / np.sqrt(D)
    o, lse = sp.sp_attn_block_fwd(q, k, v, off)
    dq, dk, dv = sp.sp_attn_block_bwd(q, k, v, o, lse, do, off)
    torch.cuda.synchronize()
    q64, k64, v64, do64 = (rn.widen_bf16(t[0]) for t in (qb, kb, vb, dob))
    o_ref, lse_ref = rb.block_attn_fwd(q64, k64, v64, scale, off)
    delta_ref = np.einsum("shd,shd->hs", o_ref, do64)
    rq, rk, rv = rb.block_attn_bwd(q64, k64, v64, lse_ref, delta_ref, do64, scale, off)
    for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        err = grad_err(host_f64(got)[0], ref)
        assert err <= GRAD_REL_L2, f"{name}: rel L2 {err:.3e}"


def test_block_step_full_size_sampled():
    """The benchmark's ring block (the 8B model's 16384-row block of all 32/8 heads against a block from the
    past).  Rows are independent in the forward, and with dO non-zero on a sampled row set only, rows outside it
    contribute nothing to any gradient: the oracle produces the sampled rows of O, LSE, dQ and ALL of dK, dV
    from those rows alone, while the kernels do the work of a dense dO."""
    n, Hq, Hkv, D = 16384, 32, 8, 128
    qb, kb, vb, dob = block_inputs(77, n, n, Hq, Hkv, D)
    rng = np.random.default_rng(3)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 255, 256, n - 257, n - 2, n - 1], rng.integers(0, n, 12)]))
    do_s = np.zeros_like(dob)
    do_s[0, rows] = dob[0, rows]
    q, k, v, do = (dev_bf16(t) for t in (qb, kb, vb, do_s))
    scale = 1.0 / np.sqrt(D)
    o, lse = sp.sp_attn_block_fwd(q, k, v, n)
    dq, dk, dv = sp.sp_attn_block_bwd(q, k, v, o, lse, do, n)
    torch.cuda.synchronize()
    q64, do64 = rn.widen_bf16(qb[0, rows]), rn.widen_bf16(do_s[0, rows])
    k64, v64 = rn.widen_bf16(kb[0]), rn.widen_bf16(vb[0])
    o_ref, lse_ref = rb.block_attn_fwd(q64, k64, v64, scale, n)
    idx = torch.from_numpy(rows).cuda()
    check_o(host_f64(o[0, idx]), o_ref, "full-size block fwd")
    assert np.abs(host_f64(lse[0][:, idx]) - lse_ref).max() <= LSE_MAX_ABS
    delta_ref = np.einsum("shd,shd->hs", o_ref, do64)
    rq, rk, rv = rb.block_attn_bwd(q64, k64, v64, lse_ref, delta_ref, do64, scale, n)
    e = (grad_err(host_f64(dq[0, idx]), rq), grad_err(host_f64(dk)[0], rk), grad_err(host_f64(dv)[0], rv))
    print(f"ring block {n}x{n}: {rows.size} active rows, rel-L2 dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert max(e) <= GRAD_REL_L2
    mask = torch.ones(n, dtype=torch.bool, device="cuda"); mask[idx] = False
    assert float(dq[0, mask].float().abs().max()) == 0.0  # rows without dO get exactly zero dQ
