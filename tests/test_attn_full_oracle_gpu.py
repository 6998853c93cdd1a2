"""Parity cases that close holes of the sampled full-size tests: the whole fp64 oracle (forward and backward,
dense dO, every element) at the 32K shard; a dense ragged multi-split length; inputs off unit variance (peaked,
near-uniform, small softmax scale); dense dO sampled at the 70B-shaped shard; the recomputed forward's bits at
128K; canaries around every output and the workspace."""
import numpy as np
import pytest
import torch

from oracle import ref_numpy as rn
from oracle import ref_stream as rs
from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import synth
from gpu_util import (GRAD_REL_L2, LSE_MAX_ABS, check_o, delta_floor, dev_bf16, grad_err, guarded, host_f64, progress)

pytestmark = pytest.mark.gpu


def gpu_fwd_bwd(q, k, v, do, scale=0.0):
    qd, kd, vd, dod = (dev_bf16(t) for t in (q, k, v, do))
    o, lse = sp.sp_attn_fwd(qd, kd, vd, softmax_scale=scale)
    dq, dk, dv = sp.sp_attn_bwd(qd, kd, vd, o, lse, dod, softmax_scale=scale)
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


@pytest.mark.timeout(900)
def test_c2_dense_dO_against_the_full_oracle():
    """S = 32768, 4 q / 1 kv heads, D = 128, dense dO: every element of O, LSE, dQ, dK and dV against the
    streaming fp64 oracle run over ALL rows and ALL key columns (3.85 TFLOP in fp64 on the host cores, in
    chunks that report progress)."""
    cfg = synth.CONFIGS["c2_8b_32k"]
    S, Hq, Hkv, D = cfg["S"], cfg["Hq"], cfg["Hkv"], cfg["D"]
    q, k, v, do = synth.attn_inputs(7, S, Hq, Hkv, D)
    o, lse, dq, dk, dv = gpu_fwd_bwd(q, k, v, do)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do))
    allr = np.arange(S)
    O = np.empty((S, Hq, D)); L = np.empty((Hq, S)); Dl = np.empty((Hq, S)); dQ = np.empty((S, Hq, D))
    nchunk = 16
    # equal-work chunks of a causal row pass: row i costs i+1 pairs
    edges = np.unique(np.round(S * np.sqrt(np.arange(nchunk + 1) / nchunk)).astype(np.int64))
    for c in range(len(edges) - 1):
        rows = allr[edges[c]:edges[c + 1]]
        r = rs.attn_rows(qf, kf, vf, rows, dof)
        O[rows] = r["O"]; L[:, rows] = r["lse"]; Dl[:, rows] = r["delta"]; dQ[rows] = r["dQ"]
        progress(f"c2 full oracle: row pass {c + 1}/{len(edges) - 1}")
    dK = np.empty((S, Hkv, D)); dV = np.empty((S, Hkv, D))
    # column j costs S-j pairs: mirror the chunking
    cedges = S - edges[::-1]
    for c in range(len(cedges) - 1):
        cols = allr[cedges[c]:cedges[c + 1]]
        dK[cols], dV[cols] = rs.attn_cols(qf, kf, vf, dof, allr, L, Dl, cols)
        progress(f"c2 full oracle: column pass {c + 1}/{len(cedges) - 1}")
    err = check_o(host_f64(o)[0], O, "c2 full")
    lerr = float(np.abs(host_f64(lse)[0] - L).max())
    e = (grad_err(host_f64(dq)[0], dQ, "dQ"), grad_err(host_f64(dk)[0], dK, "dK"), grad_err(host_f64(dv)[0], dV, "dV", abs_floor=0.0))
    print(f"c2 full oracle, dense dO: O {err:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert lerr <= LSE_MAX_ABS
    assert max(e) <= GRAD_REL_L2


def sparse_rows(S, n, seed):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 63, 64, 255, 256, S // 2, S - 257, S - 256, S - 64, S - 2, S - 1]
    return np.unique(np.concatenate([fixed, rng.integers(0, S, n)])).astype(np.int64)


def test_dense_ragged_multi_split_length():
    """S = 40037: more than 12 tiles, key tiles shared by several workgroups, and a ragged tail in every
    kernel.  Sampled rows for O/LSE/dQ; sparse dO gives the oracle all of dK, dV."""
    S, Hq, Hkv, D = 40037, 4, 1, 128
    q, k, v, do = synth.attn_inputs(8, S, Hq, Hkv, D)
    rows = sparse_rows(S, 40, 9)
    do_s = np.zeros_like(do)
    do_s[0, rows] = do[0, rows]
    o, lse, dq, dk, dv = gpu_fwd_bwd(q, k, v, do_s)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do_s))
    r = rs.attn_rows(qf, kf, vf, rows, dof)
    dk_r, dv_r = rs.attn_cols(qf, kf, vf, dof, rows, r["lse"], r["delta"], np.arange(S))
    idx = torch.from_numpy(rows).cuda()
    err = check_o(host_f64(o[0, idx]), r["O"], "ragged")
    lerr = float(np.abs(host_f64(lse[0][:, idx]) - r["lse"]).max())
    e = (grad_err(host_f64(dq[0, idx]), r["dQ"], "dQ"), grad_err(host_f64(dk)[0], dk_r, "dK"),
         grad_err(host_f64(dv)[0], dv_r, "dV", abs_floor=0.0))
    print(f"S={S}: O {err:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert lerr <= LSE_MAX_ABS and max(e) <= GRAD_REL_L2
    # dense dO on the same length: the tail window of key columns, and finiteness everywhere
    _, _, dq2, dk2, dv2 = gpu_fwd_bwd(q, k, v, do)
    W = 200
    tail = np.arange(S - W, S)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do))
    rt = rs.attn_rows(qf, kf, vf, tail, dof)
    dk_t, dv_t = rs.attn_cols(qf, kf, vf, dof, tail, rt["lse"], rt["delta"], tail)
    e2 = (grad_err(host_f64(dq2[0, S - W:]), rt["dQ"], "dQ tail"), grad_err(host_f64(dk2[0, S - W:]), dk_t, "dK tail"),
          grad_err(host_f64(dv2[0, S - W:]), dv_t, "dV tail", abs_floor=0.0))
    assert max(e2) <= GRAD_REL_L2
    for t in (dq2, dk2, dv2):
        assert torch.isfinite(t.float()).all()


def scaled_inputs(seed, S, Hq, Hkv, D, fq, fk, fv=1.0, fdo=1.0):
    """N(0,1) inputs multiplied by per-tensor factors and rounded to bf16 again (generator side only)."""
    q, k, v, do = synth.attn_inputs(seed, S, Hq, Hkv, D)
    out = []
    for t, f in ((q, fq), (k, fk), (v, fv), (do, fdo)):
        out.append(synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(t) * np.float32(f)))
    return out


RANGES = [
    # name, fq, fk, softmax_scale
    ("peaked x4", 4.0, 4.0, 0.0),                 # scores 16x larger: rows collapse onto one or two keys
    ("peaked x8", 8.0, 8.0, 0.0),                 # scores 64x larger: a row's maximum moves by more than 2^100 between tiles
    ("near-uniform", 128 ** -0.5, 128 ** -0.5, 0.0),  # inputs scaled by D^-1/2: all weights nearly equal
    ("small scale", 1.0, 1.0, 1e-3),              # LSE/scale ~ 1e4: the backward's seeds lose low bits
    ("large scale", 1.0, 1.0, 1.0),               # |s| up to ~50 without the 1/sqrt(D)
    ("lopsided", 8.0, 0.125, 0.0),                # large Q, small K
]


@pytest.mark.parametrize("name,fq,fk,scale", RANGES, ids=[r[0].replace(" ", "_") for r in RANGES])
def test_dynamic_ranges(name, fq, fk, scale):
    """Inputs off unit variance, through forward and backward, element-wise against the dense fp64 oracle:
    the lazy rescale of the forward and the -LSE/scale seed of the backward at other dynamic ranges."""
    S, Hq, Hkv, D = 2500, 4, 1, 128
    q, k, v, do = scaled_inputs(31, S, Hq, Hkv, D, fq, fk)
    o, lse, dq, dk, dv = gpu_fwd_bwd(q, k, v, do, scale)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do))
    sc = scale if scale > 0 else None
    o_r, l_r = rn.attn_fwd(qf, kf, vf, sc)
    dq_r, dk_r, dv_r, _ = rn.attn_bwd(qf, kf, vf, dof, sc)
    err = check_o(host_f64(o)[0], o_r, name, big_from=2.0 if name in ("peaked x4", "peaked x8", "large scale") else 4.0)
    # LSE bar scales with its magnitude here (fp32: 2^-23 relative per operation on values up to |LSE|)
    lerr = float(np.abs(host_f64(lse)[0] - l_r).max())
    lbar = max(LSE_MAX_ABS, 4e-6 * float(np.abs(l_r).max()))
    rms = lambda x: float(np.sqrt(np.mean(x * x)))
    sc_eff = scale if scale > 0 else 1.0 / np.sqrt(D)
    fl_q = delta_floor(sc_eff, D, rms(dof), rms(vf), float(np.linalg.norm(kf, axis=-1).max()))
    fl_k = delta_floor(sc_eff, D, rms(dof), rms(vf), float(np.linalg.norm(qf, axis=-1).max()))
    e = (grad_err(host_f64(dq)[0], dq_r, "dQ", abs_floor=fl_q), grad_err(host_f64(dk)[0], dk_r, "dK", abs_floor=fl_k),
         grad_err(host_f64(dv)[0], dv_r, "dV", abs_floor=0.0))
    print(f"{name}: max|LSE| {np.abs(l_r).max():.1f}; O {err:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert lerr <= lbar, (lerr, lbar)
    assert max(e) <= GRAD_REL_L2, e
    for t in (o, dq, dk, dv):
        assert torch.isfinite(t.float()).all()


def test_c4_dense_dO_sampled():
    """70B-shaped shard (8 q / 1 kv at 128K) with dense dO: sampled dQ rows, the tail window of key columns,
    sum_j dV_j = sum_i dO_i."""
    cfg = synth.CONFIGS["c4_70b_128k"]
    S, Hq, Hkv, D = cfg["S"], cfg["Hq"], cfg["Hkv"], cfg["D"]
    q, k, v, do = synth.attn_inputs(2, S, Hq, Hkv, D)
    _, _, dq, dk, dv = gpu_fwd_bwd(q, k, v, do)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do))
    rows = sparse_rows(S, 12, 5)
    r = rs.attn_rows(qf, kf, vf, rows, dof)
    e_dq = grad_err(host_f64(dq[0, torch.from_numpy(rows).cuda()]), r["dQ"], "dQ")
    W = 160
    tail = np.arange(S - W, S)
    rt = rs.attn_rows(qf, kf, vf, tail, dof)
    dk_r, dv_r = rs.attn_cols(qf, kf, vf, dof, tail, rt["lse"], rt["delta"], tail)
    e_dk = grad_err(host_f64(dk[0, S - W:]), dk_r, "dK tail")
    e_dv = grad_err(host_f64(dv[0, S - W:]), dv_r, "dV tail", abs_floor=0.0)
    print(f"c4 dense dO: dQ(sampled) {e_dq:.2e} dK(tail) {e_dk:.2e} dV(tail) {e_dv:.2e}")
    assert max(e_dq, e_dk, e_dv) <= GRAD_REL_L2
    want = dof.reshape(S, Hkv, Hq // Hkv, D).sum(axis=(0, 2))
    got = dv[0].double().sum(dim=0).cpu().numpy()
    assert np.abs(got - want).max() <= 0.01 * np.sqrt(S * Hq / Hkv)
    for t in (dq, dk, dv):
        assert torch.isfinite(t.float()).all()


OTHER_SHARDS = [
    # the head shards at P = 8 of the other models of Section 4's setup, at the length the benchmark times them
    ("llama3.2-1b", 65536, 4, 1, 64),    # head dim 64
    ("llama2-13b", 65536, 5, 5, 128),    # full attention: every query head has its own key/value head
    ("llama3.2-3b", 65536, 3, 1, 128),   # three query heads on one key/value head
]


@pytest.mark.parametrize("name,S,Hq,Hkv,D", OTHER_SHARDS, ids=[t[0] for t in OTHER_SHARDS])
def test_other_model_shards_full_size(name, S, Hq, Hkv, D):
    """Full-size head shards of the other evaluated models: sampled rows of O, LSE and dQ, and with dO
    non-zero on the sampled rows only, all of dK and dV."""
    q, k, v, do = synth.attn_inputs(13, S, Hq, Hkv, D)
    rows = sparse_rows(S, 24, 6)
    do_s = np.zeros_like(do)
    do_s[0, rows] = do[0, rows]
    o, lse, dq, dk, dv = gpu_fwd_bwd(q, k, v, do_s)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do_s))
    r = rs.attn_rows(qf, kf, vf, rows, dof)
    dk_r, dv_r = rs.attn_cols(qf, kf, vf, dof, rows, r["lse"], r["delta"], np.arange(S))
    idx = torch.from_numpy(rows).cuda()
    err = check_o(host_f64(o[0, idx]), r["O"], name)
    lerr = float(np.abs(host_f64(lse[0][:, idx]) - r["lse"]).max())
    e = (grad_err(host_f64(dq[0, idx]), r["dQ"], "dQ"), grad_err(host_f64(dk)[0], dk_r, "dK"),
         grad_err(host_f64(dv)[0], dv_r, "dV", abs_floor=0.0))
    print(f"{name}: O {err:.2e} LSE {lerr:.2e} dQ {e[0]:.2e} dK {e[1]:.2e} dV {e[2]:.2e}")
    assert lerr <= LSE_MAX_ABS and max(e) <= GRAD_REL_L2
    # dense dO: the tail window of key columns, every gradient finite
    _, _, dq2, dk2, dv2 = gpu_fwd_bwd(q, k, v, do)
    W = 160
    tail = np.arange(S - W, S)
    qf, kf, vf, dof = (rn.widen_bf16(t[0]) for t in (q, k, v, do))
    rt = rs.attn_rows(qf, kf, vf, tail, dof)
    dk_t, dv_t = rs.attn_cols(qf, kf, vf, dof, tail, rt["lse"], rt["delta"], tail)
    e2 = (grad_err(host_f64(dq2[0, S - W:]), rt["dQ"], "dQ tail"), grad_err(host_f64(dk2[0, S - W:]), dk_t, "dK tail"),
          grad_err(host_f64(dv2[0, S - W:]), dv_t, "dV tail", abs_floor=0.0))
    assert max(e2) <= GRAD_REL_L2
    for t in (dq2, dk2, dv2):
        assert torch.isfinite(t.float()).all()


def test_recompute_forward_is_bitwise_the_first_forward_at_128k():
    """Checkpoint-recompute (Section 3.2) runs the forward a second time in the backward pass: at the 128K
    shard the second run gives the first run's bits (fresh output buffers, other work in between)."""
    cfg = synth.CONFIGS["c3_8b_128k"]
    S, Hq, Hkv, D = cfg["S"], cfg["Hq"], cfg["Hkv"], cfg["D"]
    q, k, v, do = synth.attn_inputs(3, S, Hq, Hkv, D)
    qd, kd, vd, dod = (dev_bf16(t) for t in (q, k, v, do))
    o1, l1 = sp.sp_attn_fwd(qd, kd, vd)
    dq, dk, dv = sp.sp_attn_bwd(qd, kd, vd, o1, l1, dod)  # something else on the device in between
    o2 = torch.full_like(o1, float("nan")); l2 = torch.full_like(l1, float("nan"))
    sp.sp_attn_fwd(qd, kd, vd, o=o2, lse=l2)
    dq2, dk2, dv2 = sp.sp_attn_bwd(qd, kd, vd, o2, l2, dod)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    assert torch.equal(l1.view(torch.int32), l2.view(torch.int32))
    for a, b in ((dq, dq2), (dk, dk2), (dv, dv2)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_guard_regions_dense_ragged():
    """Canaries in front of and behind O, LSE, dQ, dK, dV and the backward workspace at ragged extents
    (B = 2, S = 1000 and a one-row problem): no kernel writes a byte outside what the header says it owns."""
    for (B, S, Hq, Hkv, D) in ((2, 1000, 4, 1, 128), (1, 2100, 2, 2, 64), (1, 1, 2, 1, 128)):
        q, k, v, do = synth.attn_inputs(41 + S, S, Hq, Hkv, D, B)
        qd, kd, vd, dod = (dev_bf16(t) for t in (q, k, v, do))
        bf = torch.bfloat16
        o, c_o = guarded((B, S, Hq, D), bf); lse, c_l = guarded((B, Hq, S), torch.float32)
        dq, c_dq = guarded((B, S, Hq, D), bf); dk, c_dk = guarded((B, S, Hkv, D), bf); dv, c_dv = guarded((B, S, Hkv, D), bf)
        nws = sp.sp_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D)
        ws, c_ws = guarded((nws,), torch.uint8)
        sp.sp_attn_fwd(qd, kd, vd, o=o, lse=lse)
        sp.sp_attn_bwd(qd, kd, vd, o, lse, dod, dq=dq, dk=dk, dv=dv, workspace=ws)
        for c, n in ((c_o, "O"), (c_l, "LSE"), (c_dq, "dQ"), (c_dk, "dK"), (c_dv, "dV"), (c_ws, "workspace")):
            c(f"{n} at B={B} S={S}")
        # and the guarded run is the ordinary run
        o2, l2 = sp.sp_attn_fwd(qd, kd, vd)
        g2 = sp.sp_attn_bwd(qd, kd, vd, o2, l2, dod)
        torch.cuda.synchronize()
        assert torch.equal(o.view(torch.int16), o2.view(torch.int16)) and torch.equal(lse, l2)
        for a, b in zip((dq, dk, dv), g2):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_guard_regions_packed_documents():
    lengths = [130, 0, 64, 1, 300, 63, 129, 2040, 8, 30, 2]
    cu = synth.cu_seqlens_from_lengths(lengths)
    T, Hq, Hkv, D = int(cu[-1]), 4, 1, 128
    q, k, v, do = synth.attn_inputs(43, T, Hq, Hkv, D)
    qd, kd, vd, dod = (dev_bf16(t[0]) for t in (q, k, v, do))
    cud = torch.from_numpy(cu).cuda()
    bf = torch.bfloat16
    o, c_o = guarded((T, Hq, D), bf); lse, c_l = guarded((Hq, T), torch.float32)
    dq, c_dq = guarded((T, Hq, D), bf); dk, c_dk = guarded((T, Hkv, D), bf); dv, c_dv = guarded((T, Hkv, D), bf)
    wf, c_wf = guarded((sp.sp_attn_varlen_fwd_workspace_bytes(T, Hq, Hkv, D, len(lengths)),), torch.uint8)
    wb, c_wb = guarded((sp.sp_attn_bwd_workspace_bytes(1, T, Hq, Hkv, D, len(lengths)),), torch.uint8)
    sp.sp_attn_varlen_fwd(qd, kd, vd, cud, o=o, lse=lse, workspace=wf)
    sp.sp_attn_varlen_bwd(qd, kd, vd, o, lse, dod, cud, dq=dq, dk=dk, dv=dv, workspace=wb)
    for c, n in ((c_o, "O"), (c_l, "LSE"), (c_dq, "dQ"), (c_dk, "dK"), (c_dv, "dV"), (c_wf, "fwd workspace"),
                 (c_wb, "bwd workspace")):
        c(n)
    o2, l2 = sp.sp_attn_varlen_fwd(qd, kd, vd, cud)
    g2 = sp.sp_attn_varlen_bwd(qd, kd, vd, o2, l2, dod, cud)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), o2.view(torch.int16)) and torch.equal(lse, l2)
    for a, b in zip((dq, dk, dv), g2):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
