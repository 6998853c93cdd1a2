"""Parity of the packed variable-length (block-diagonal causal) entry points."""
import numpy as np
import pytest
import torch

from oracle import ref_numpy as rn
from oracle import ref_stream as rs
from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import synth
from gpu_util import GRAD_REL_L2, LSE_MAX_ABS, check_o, dev_bf16, host_f64, grad_err

pytestmark = pytest.mark.gpu


def run_varlen(q, k, v, do, cu, scale=0.0):
    qd, kd, vd, dod = (dev_bf16(t[0]) for t in (q, k, v, do))
    cud = torch.from_numpy(np.asarray(cu, np.int32)).cuda()
    o, lse = sp.sp_attn_varlen_fwd(qd, kd, vd, cud, softmax_scale=scale)
    dq, dk, dv = sp.sp_attn_varlen_bwd(qd, kd, vd, o, lse, dod, cud, softmax_scale=scale)
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


CASES = [
    # lengths, Hq, Hkv, D
    ([5, 0, 17, 1, 9], 4, 2, 64),                 # tiny docs, an empty one
    ([130, 64, 1, 300, 63, 129], 4, 1, 128),      # boundaries off every tile edge
    ([1000], 2, 1, 128),                          # one document
    ([0, 0, 257, 0, 128, 128, 0], 2, 2, 64),      # leading/trailing empties, aligned docs
    ([700, 900, 333], 8, 2, 128),
    ([2040, 8, 30, 2], 4, 1, 128),                # last key tile has fewer steps than workgroups sharing it
]


@pytest.mark.parametrize("lengths,Hq,Hkv,D", CASES)
def test_varlen_matches_oracle(lengths, Hq, Hkv, D):
    cu = synth.cu_seqlens_from_lengths(lengths)
    T = int(cu[-1])
    q, k, v, do = synth.attn_inputs(T + len(lengths), T, Hq, Hkv, D)
    o, lse, dq, dk, dv = run_varlen(q, k, v, do, cu)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do))
    o_r, l_r = rn.attn_varlen_fwd(qf, kf, vf, cu)
    dq_r, dk_r, dv_r, _ = rn.attn_varlen_bwd(qf, kf, vf, dof, cu)
    err = check_o(host_f64(o), o_r)
    lerr = np.abs(host_f64(lse) - l_r).max()
    e = (grad_err(host_f64(dq), dq_r), grad_err(host_f64(dk), dk_r), grad_err(host_f64(dv), dv_r))
    print(f"lengths={lengths}: O {err:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert lerr <= LSE_MAX_ABS
    assert max(e) <= GRAD_REL_L2


def test_varlen_single_document_equals_dense_bitwise():
    S, Hq, Hkv, D = 900, 4, 1, 128
    q, k, v, do = synth.attn_inputs(21, S, Hq, Hkv, D)
    o, lse, dq, dk, dv = run_varlen(q, k, v, do, [0, S])
    qd, kd, vd, dod = (dev_bf16(t) for t in (q, k, v, do))
    o2, lse2 = sp.sp_attn_fwd(qd, kd, vd)
    dq2, dk2, dv2 = sp.sp_attn_bwd(qd, kd, vd, o2, lse2, dod)
    for a, b in ((o, o2[0]), (dq, dq2[0]), (dk, dk2[0]), (dv, dv2[0])):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.equal(lse, lse2[0])


def test_varlen_documents_do_not_leak():
    """Poison one document (huge K/V/Q/dO); the others must come out bit-identical."""
    lengths = [100, 77, 200]
    cu = synth.cu_seqlens_from_lengths(lengths)
    T = int(cu[-1])
    Hq, Hkv, D = 4, 2, 128
    q, k, v, do = synth.attn_inputs(22, T, Hq, Hkv, D)
    base = run_varlen(q, k, v, do, cu)
    q2, k2, v2, do2 = q.copy(), k.copy(), v.copy(), do.copy()
    big = synth.f32_to_bf16_bits(np.array([3e4], np.float32))[0]
    for t in (q2, k2, v2, do2):
        t[0, 100:177] = big
    pois = run_varlen(q2, k2, v2, do2, cu)
    keep = torch.from_numpy(np.r_[0:100, 177:T]).cuda()
    for a, b in zip(base, pois):
        if a.dim() == 2:  # lse [Hq, T]
            assert torch.equal(a[:, keep], b[:, keep])
        else:
            assert torch.equal(a[keep].view(torch.int16), b[keep].view(torch.int16))


@pytest.mark.parametrize("T,seed", [(65536, 0), (90112 + 77, 5)])
def test_varlen_full_size_workload(T, seed):
    """T = 65536 packed documents with lognormal lengths (the benchmark's workload), and a longer, ragged batch
    with more than 256 tiles for the kernels that order them: sampled rows for the forward and dQ, sparse dO
    for all of dK/dV."""
    cfg = synth.CONFIGS["c5_varlen_64k"]
    assert cfg["T"] == 65536
    Hq, Hkv, D = cfg["Hq"], cfg["Hkv"], cfg["D"]
    lengths = synth.doc_lengths(seed, T)
    cu = synth.cu_seqlens_from_lengths(lengths)
    q, k, v, do = synth.attn_inputs(0, T, Hq, Hkv, D)
    rng = np.random.default_rng(4)
    edges = np.concatenate([cu[:-1], cu[1:] - 1, cu[:-1] + 1])
    rows = np.unique(np.clip(np.concatenate([edges, rng.integers(0, T, 64)]), 0, T - 1)).astype(np.int64)
    do_s = np.zeros_like(do)
    do_s[0, rows] = do[0, rows]
    o, lse, dq, dk, dv = run_varlen(q, k, v, do_s, cu)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do_s))
    r = rs.attn_rows(qf, kf, vf, rows, dof, cu_seqlens=cu)
    dk_r, dv_r = rs.attn_cols(qf, kf, vf, dof, rows, r["lse"], r["delta"], np.arange(T), cu_seqlens=cu)
    idx = torch.from_numpy(rows).cuda()
    err = check_o(host_f64(o[idx]), r["O"])
    lerr = np.abs(host_f64(lse[:, idx]) - r["lse"]).max()
    e = (grad_err(host_f64(dq[idx]), r["dQ"]), grad_err(host_f64(dk), dk_r), grad_err(host_f64(dv), dv_r))
    print(f"varlen T={T} ({len(lengths)} docs): O {err:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert lerr <= LSE_MAX_ABS and max(e) <= GRAD_REL_L2


@pytest.mark.parametrize("hint", [0, 1, 700, 4000, 10**9])
def test_varlen_max_seqlen_is_only_a_hint(hint):
    """max_seqlen shapes the backward's work split and nothing else: exact, too small, too large or absent,
    the results stay within the parity bars (the forward does not depend on it at all)."""
    lengths = [700, 1500, 333, 1467]
    cu = synth.cu_seqlens_from_lengths(lengths)
    T, Hq, Hkv, D = int(cu[-1]), 4, 1, 128
    q, k, v, do = synth.attn_inputs(91, T, Hq, Hkv, D)
    qd, kd, vd, dod = (dev_bf16(t[0]) for t in (q, k, v, do))
    cud = torch.from_numpy(np.asarray(cu, np.int32)).cuda()
    o0, lse0 = sp.sp_attn_varlen_fwd(qd, kd, vd, cud)
    o, lse = sp.sp_attn_varlen_fwd(qd, kd, vd, cud, max_seqlen=min(hint, 2**31 - 1))
    assert torch.equal(o.view(torch.int16), o0.view(torch.int16)) and torch.equal(lse, lse0)
    dq, dk, dv = sp.sp_attn_varlen_bwd(qd, kd, vd, o, lse, dod, cud, max_seqlen=min(hint, 2**31 - 1))
    torch.cuda.synchronize()
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do))
    dq_r, dk_r, dv_r, _ = rn.attn_varlen_bwd(qf, kf, vf, dof, cu)
    e = (grad_err(host_f64(dq), dq_r), grad_err(host_f64(dk), dk_r), grad_err(host_f64(dv), dv_r))
    assert max(e) <= GRAD_REL_L2, e


def test_cu_seqlens_check_kernel():
    """The debug check of a cu_seqlens array: well formed, wrong start, decreasing, wrong end, and all three."""
    cases = [([0, 5, 5, 17, 300], 300, 0), ([1, 5, 300], 300, 1), ([0, 200, 100, 300], 300, 2), ([0, 100, 299], 300, 4),
             ([3, 2, 1], 300, 7), ([0], 0, 0), (list(range(0, 70001, 7)), 70000, 0),
             (list(range(0, 70001, 7))[:5000] + [1] + list(range(0, 70001, 7))[5001:], 70000, 2)]
    for cu, T, want in cases:
        flag = sp.sp_varlen_check_cu_seqlens(torch.tensor(cu, dtype=torch.int32, device="cuda"), T)
        torch.cuda.synchronize()
        assert int(flag.item()) == want, (cu[:6], T, int(flag.item()), want)
