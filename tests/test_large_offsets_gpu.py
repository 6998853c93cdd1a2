"""Tensors past 2^32 elements: every kernel's address arithmetic has to be 64-bit.

The batch entries checked sit past element 2^31 and past element 2^32 of the
query-side tensors, so an offset that wrapped at either width would read or write
another entry (their contents differ: one device random stream over the whole
tensor)."""
import numpy as np
import pytest
import torch

from oracle import ref_numpy as rn
from oracle import ref_stream as rs
from paper_2604_27089_amd import binding as sp
from gpu_util import GRAD_REL_L2, LSE_MAX_ABS, check_o, grad_err, host_bits, host_f64, progress

pytestmark = pytest.mark.gpu


def test_attention_batch_past_2_to_32_elements():
    B, S, Hq, Hkv, D = 2176, 2048, 8, 2, 128
    assert B * S * Hq * D > 2 ** 32 and B * S * Hkv * D > 2 ** 30
    g = torch.Generator(device="cuda").manual_seed(20)
    bf = dict(dtype=torch.bfloat16, device="cuda")
    q, do = (torch.empty((B, S, Hq, D), **bf).normal_(generator=g) for _ in range(2))
    k, v = (torch.empty((B, S, Hkv, D), **bf).normal_(generator=g) for _ in range(2))
    progress(f"large batch: inputs on the device ({4 * q.numel() * 2 / 2**30:.1f} GiB query-side)")
    o, lse = sp.sp_attn_fwd(q, k, v)
    dq, dk, dv = sp.sp_attn_bwd(q, k, v, o, lse, do)
    torch.cuda.synchronize()
    progress("large batch: forward and backward done")
    per_entry = S * Hq * D
    picks = (0, 2 ** 31 // per_entry + 76, B - 1)
    assert picks[1] * per_entry > 2 ** 31 and picks[2] * per_entry > 2 ** 32
    for b in picks:
        qh, kh, vh, doh = (rn.widen_bf16(host_bits(t[b])) for t in (q, k, v, do))
        o_r, lse_r = rs.attn_fwd(qh, kh, vh)
        # the backward's Delta comes from the bf16 O the kernels saw; the oracle uses its own exact O
        dq_r, dk_r, dv_r, _ = rs.attn_bwd(qh, kh, vh, doh)
        oerr = check_o(host_f64(o[b]), o_r, f"b={b}")
        lerr = float(np.abs(host_f64(lse[b]) - lse_r).max())
        e = [grad_err(host_f64(dq[b]), dq_r, f"dQ b={b}"), grad_err(host_f64(dk[b]), dk_r, f"dK b={b}"),
             grad_err(host_f64(dv[b]), dv_r, f"dV b={b}", abs_floor=0.0)]
        progress(f"large batch b={b}: O {oerr:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
        assert lerr <= LSE_MAX_ABS and max(e) <= GRAD_REL_L2


@pytest.mark.parametrize("B,S_l", [(1, 2 ** 19), (2, 2 ** 18)])
def test_relayout_past_2_to_32_elements(B, S_l):
    H, D, P = 64, 128, 8
    assert B * S_l * H * D == 2 ** 32
    g = torch.Generator(device="cuda").manual_seed(21)
    x = torch.randint(-32768, 32767, (B, S_l, H, D), dtype=torch.int16, device="cuda", generator=g)
    y = sp.sp_pack_seq_to_head(x, P)
    back = sp.sp_unpack_head_to_seq(y, P)
    assert y.shape == (B, P * S_l, H // P, D)
    assert torch.equal(back, x)
    del back
    rng = np.random.default_rng(1)
    h = H // P
    for b in range(B):
        for p in range(P):
            for s in [0, S_l - 1] + [int(t) for t in rng.integers(0, S_l, 6)]:
                # the index map, row by row: out[b, p*S_l + s, j, :] = in[b, s, p*h + j, :]
                assert np.array_equal(y[b, p * S_l + s].cpu().numpy(), x[b, s, p * h:(p + 1) * h].cpu().numpy())


def test_packed_documents_past_2_to_32_elements():
    """4.2 million packed rows: more tiles than the longest-first ordering ranks (the kernels then take the
    tiles in plain order), query-side tensors past 2^32 elements; the first document, one past element 2^31
    and the last against the oracle on that document alone."""
    from paper_2604_27089_amd import synth
    T, Hq, Hkv, D = 2 ** 22 + 777, 8, 2, 128
    assert T * Hq * D > 2 ** 32 and (T + 255) // 256 > 16384
    lengths = synth.doc_lengths(3, T, mean=2048.0, hi=4096)
    cu = synth.cu_seqlens_from_lengths(lengths)
    g = torch.Generator(device="cuda").manual_seed(22)
    bf = dict(dtype=torch.bfloat16, device="cuda")
    q, do = (torch.empty((T, Hq, D), **bf).normal_(generator=g) for _ in range(2))
    k, v = (torch.empty((T, Hkv, D), **bf).normal_(generator=g) for _ in range(2))
    cud = torch.from_numpy(np.asarray(cu, np.int32)).cuda()
    progress(f"large packed batch: {len(lengths)} documents, longest {max(lengths)}")
    o, lse = sp.sp_attn_varlen_fwd(q, k, v, cud, max_seqlen=max(lengths))
    dq, dk, dv = sp.sp_attn_varlen_bwd(q, k, v, o, lse, do, cud, max_seqlen=max(lengths))
    torch.cuda.synchronize()
    progress("large packed batch: forward and backward done")
    mid = int(np.searchsorted(cu, 2 ** 31 // (Hq * D) + 5000, side="right"))
    assert int(cu[mid]) * Hq * D > 2 ** 31
    for d in (0, mid, len(lengths) - 1):
        a, b = int(cu[d]), int(cu[d + 1])
        qh, kh, vh, doh = (rn.widen_bf16(host_bits(t[a:b])) for t in (q, k, v, do))
        o_r, lse_r = rs.attn_fwd(qh, kh, vh)
        dq_r, dk_r, dv_r, _ = rs.attn_bwd(qh, kh, vh, doh)
        oerr = check_o(host_f64(o[a:b]), o_r, f"doc {d}")
        lerr = float(np.abs(host_f64(lse[:, a:b]) - lse_r).max())
        e = [grad_err(host_f64(dq[a:b]), dq_r, f"dQ doc {d}"), grad_err(host_f64(dk[a:b]), dk_r, f"dK doc {d}"),
             grad_err(host_f64(dv[a:b]), dv_r, f"dV doc {d}", abs_floor=0.0)]
        progress(f"large packed batch doc {d} rows [{a},{b}): O {oerr:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
        assert lerr <= LSE_MAX_ABS and max(e) <= GRAD_REL_L2


def test_sequence_of_half_a_million_rows():
    """One sequence four times the longest configured one, ragged: 2050 query tiles and key tiles per head,
    8199 key steps for the last rows.  Sampled rows for O, LSE and dQ; dO lives on the sampled rows only, so
    the oracle gives all of dK and dV from them while the kernels do a dense backward's work."""
    S, Hq, Hkv, D = 2 ** 19 + 421, 2, 1, 128
    g = torch.Generator(device="cuda").manual_seed(23)
    bf = dict(dtype=torch.bfloat16, device="cuda")
    qd, do_full = (torch.empty((1, S, Hq, D), **bf).normal_(generator=g) for _ in range(2))
    kd, vd = (torch.empty((1, S, Hkv, D), **bf).normal_(generator=g) for _ in range(2))
    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, S - 422, S - 421, S - 2, S - 1], rng.integers(0, S, 12)])).astype(np.int64)
    idx = torch.from_numpy(rows).cuda()
    dod = torch.zeros_like(do_full)
    dod[0, idx] = do_full[0, idx]
    del do_full
    progress(f"long sequence: S = {S}, inputs on the device")
    o, lse = sp.sp_attn_fwd(qd, kd, vd)
    dq, dk, dv = sp.sp_attn_bwd(qd, kd, vd, o, lse, dod)
    torch.cuda.synchronize()
    progress("long sequence: forward and backward done")
    qf, kf, vf, dof = (rn.widen_bf16(host_bits(t[0])) for t in (qd, kd, vd, dod))
    r = rs.attn_rows(qf, kf, vf, rows, dof)
    dk_r, dv_r = rs.attn_cols(qf, kf, vf, dof, rows, r["lse"], r["delta"], np.arange(S))
    oerr = check_o(host_f64(o[0, idx]), r["O"], "long sequence")
    lerr = float(np.abs(host_f64(lse[0][:, idx]) - r["lse"]).max())
    e = [grad_err(host_f64(dq[0, idx]), r["dQ"], "dQ"), grad_err(host_f64(dk)[0], dk_r, "dK"),
         grad_err(host_f64(dv)[0], dv_r, "dV", abs_floor=0.0)]
    progress(f"long sequence: O {oerr:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert lerr <= LSE_MAX_ABS and max(e) <= GRAD_REL_L2
    mask = torch.ones(S, dtype=torch.bool, device="cuda"); mask[idx] = False
    assert float(dq[0, mask].float().abs().max()) == 0.0  # rows without dO get exactly zero dQ
