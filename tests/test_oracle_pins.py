"""Pins of the CPU oracle against things other than itself: brute force,
closed forms, invariants, library routines (torch fp64 autograd, scipy),
finite differences, a hand-worked fixture and the simulated P-rank Ulysses
data flow.  CPU only."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import ref_numpy as rn
from oracle import ref_stream as rs
from paper_2604_27089_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_qkv(seed, S, Hq, Hkv, D):
    q, k, v, do = synth.attn_inputs(seed, S, Hq, Hkv, D)
    return tuple(rn.widen_bf16(t)[0] for t in (q, k, v, do))


# ------------------------------------------------------------------ re-layout
def test_relayout_hand_worked_fixture():
    vals = {}
    for line in open(os.path.join(GOLDEN, "relayout_worked_example.txt")):
        if line.startswith("#") or ":" not in line:
            continue
        key, rest = line.split(":")
        vals[key.strip()] = np.array(rest.split(), dtype=np.uint16)
    x = vals["in"].reshape(2, 4, 1)
    for fn in (rn.pack_seq_to_head, rn.pack_seq_to_head_loops):
        assert np.array_equal(fn(x, 2).ravel(), vals["out"])
    assert np.array_equal(rs.pack_seq_to_head(x[None], 2).ravel(), vals["out"])
    y = vals["out"].reshape(4, 2, 1)
    for fn in (rn.unpack_head_to_seq, rn.unpack_head_to_seq_loops):
        assert np.array_equal(fn(y, 2).ravel(), vals["in"])
    assert np.array_equal(rs.unpack_head_to_seq(y[None], 2).ravel(), vals["in"])


@pytest.mark.parametrize("S_l,H,D,P", [(6, 8, 4, 4), (5, 6, 3, 3), (7, 4, 8, 1), (3, 8, 2, 8)])
def test_relayout_three_writings_agree_and_invert(S_l, H, D, P):
    x = synth.pack_input(1, 2, S_l, H, D)
    for b in range(2):
        a = rn.pack_seq_to_head(x[b], P)
        assert np.array_equal(a, rn.pack_seq_to_head_loops(x[b], P))
        assert np.array_equal(rn.unpack_head_to_seq(a, P), x[b])
        assert np.array_equal(rn.unpack_head_to_seq_loops(a, P), x[b])
        assert np.array_equal(rn.pack_seq_to_head(rn.unpack_head_to_seq(a, P), P), a)
    c = rs.pack_seq_to_head(x, P)
    assert np.array_equal(c, np.stack([rn.pack_seq_to_head(x[b], P) for b in range(2)]))
    assert np.array_equal(rs.unpack_head_to_seq(c, P), x)
    if P == 1:
        assert np.array_equal(c.reshape(x.shape), x)
    # 4-byte elements travel the same way
    x4 = ((np.arange(S_l * H * D, dtype=np.uint64) * 2654435761) % (1 << 32)).astype(np.uint32)
    x4 = x4.reshape(1, S_l, H, D)
    assert np.array_equal(rs.unpack_head_to_seq(rs.pack_seq_to_head(x4, P), P), x4)
    assert np.array_equal(rs.pack_seq_to_head(x4, P)[0], rn.pack_seq_to_head(x4[0], P))


def simulate_all_to_all(chunks_per_rank):
    """chunks_per_rank[r][p] = what rank r sends to rank p; returns recv[p][r]."""
    P = len(chunks_per_rank)
    return [[chunks_per_rank[r][p] for r in range(P)] for p in range(P)]


@pytest.mark.parametrize("P,S,H,D", [(4, 16, 8, 4), (2, 10, 6, 2)])
def test_relayout_simulated_ranks_reassemble_head_shard(P, S, H, D):
    """After pack + exchange, rank p holds X[:, p*h:(p+1)*h, :] of the global
    activation (whole sequence, its heads): Section 2's description."""
    X = synth.pack_input(3, 1, S, H, D)[0]
    S_l, h = S // P, H // P
    sends = []
    for r in range(P):
        packed = rn.pack_seq_to_head(X[r * S_l:(r + 1) * S_l], P)
        sends.append([packed[p * S_l:(p + 1) * S_l] for p in range(P)])
    recv = simulate_all_to_all(sends)
    for p in range(P):
        got = np.concatenate(recv[p], axis=0)  # source ranks in order = sequence order
        assert np.array_equal(got, X[:, p * h:(p + 1) * h, :])
    # and back: every rank splits its [S,h,D] by destination rank's token range,
    # the receiver lays the P pieces out chunk-major and unpacks.
    sends_back = [[X[r * S_l:(r + 1) * S_l, p * h:(p + 1) * h, :] for r in range(P)] for p in range(P)]
    recv_back = simulate_all_to_all(sends_back)
    for r in range(P):
        chunked = np.concatenate(recv_back[r], axis=0)  # [P*S_l, h, D]
        assert np.array_equal(rn.unpack_head_to_seq(chunked, P), X[r * S_l:(r + 1) * S_l])


# ------------------------------------------------------------ attention forward
def brute_force_fwd(q, k, v, scale, G):
    """Pure-Python triple loop, written independently of the oracle."""
    S, Hq, D = q.shape
    o = np.zeros((S, Hq, D)); lse = np.zeros((Hq, S))
    for a in range(Hq):
        g = a // G
        for i in range(S):
            sc = [scale * sum(q[i, a, d] * k[j, g, d] for d in range(D)) for j in range(i + 1)]
            mx = max(sc)
            z = sum(math.exp(x - mx) for x in sc)
            lse[a, i] = mx + math.log(z)
            for j in range(i + 1):
                w = math.exp(sc[j] - mx) / z
                for d in range(D):
                    o[i, a, d] += w * v[j, g, d]
    return o, lse


@pytest.mark.parametrize("S,Hq,Hkv,D", [(9, 2, 1, 4), (17, 4, 2, 8), (12, 3, 3, 5)])
def test_fwd_brute_force(S, Hq, Hkv, D):
    q, k, v, _ = rand_qkv(0, S, Hq, Hkv, D)
    scale = 0.37
    o_b, l_b = brute_force_fwd(q, k, v, scale, Hq // Hkv)
    o_n, l_n = rn.attn_fwd(q, k, v, scale)
    o_c, l_c = rs.attn_fwd(q, k, v, softmax_scale=scale)
    for o, l in ((o_n, l_n), (o_c, l_c)):
        np.testing.assert_allclose(o, o_b, rtol=0, atol=1e-13)
        np.testing.assert_allclose(l, l_b, rtol=0, atol=1e-13)


def torch_reference(q, k, v, do, scale, G):
    """Composed torch fp64 ops + autograd: an independent library route."""
    tq, tk, tv = (torch.tensor(t, dtype=torch.float64, requires_grad=True) for t in (q, k, v))
    S = q.shape[0]
    kk = tk.repeat_interleave(G, dim=1); vv = tv.repeat_interleave(G, dim=1)
    s = torch.einsum("iad,jad->aij", tq, kk) * scale
    mask = torch.ones(S, S, dtype=torch.bool).tril()
    s = s.masked_fill(~mask, float("-inf"))
    lse = torch.logsumexp(s, dim=-1)
    o = torch.einsum("aij,jad->iad", torch.softmax(s, dim=-1), vv)
    (o * torch.tensor(do)).sum().backward()
    return o.detach().numpy(), lse.detach().numpy(), tq.grad.numpy(), tk.grad.numpy(), tv.grad.numpy()


@pytest.mark.parametrize("S,Hq,Hkv,D", [(33, 4, 1, 16), (64, 2, 2, 8), (50, 6, 2, 12)])
def test_fwd_bwd_against_torch_autograd_fp64(S, Hq, Hkv, D):
    q, k, v, do = rand_qkv(1, S, Hq, Hkv, D)
    scale = 1.0 / math.sqrt(D)
    o_t, l_t, dq_t, dk_t, dv_t = torch_reference(q, k, v, do, scale, Hq // Hkv)
    o_n, l_n = rn.attn_fwd(q, k, v)            # default scale = 1/sqrt(D)
    dq_n, dk_n, dv_n, _ = rn.attn_bwd(q, k, v, do)
    o_c, l_c = rs.attn_fwd(q, k, v)
    dq_c, dk_c, dv_c, _ = rs.attn_bwd(q, k, v, do)
    for got, ref in ((o_n, o_t), (l_n, l_t), (dq_n, dq_t), (dk_n, dk_t), (dv_n, dv_t),
                     (o_c, o_t), (l_c, l_t), (dq_c, dq_t), (dk_c, dk_t), (dv_c, dv_t)):
        np.testing.assert_allclose(got, ref, rtol=0, atol=2e-12)


def test_fwd_sdpa_library_routine():
    S, Hq, Hkv, D = 40, 4, 2, 16
    q, k, v, _ = rand_qkv(2, S, Hq, Hkv, D)
    tq, tk, tv = (torch.tensor(t).permute(1, 0, 2)[None] for t in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq, tk.repeat_interleave(2, dim=1), tv.repeat_interleave(2, dim=1), is_causal=True)
    ref = ref[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(rn.attn_fwd(q, k, v)[0], ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(rs.attn_fwd(q, k, v)[0], ref, rtol=0, atol=1e-12)


def test_fwd_scipy_softmax_row():
    S, D = 21, 8
    q, k, v, _ = rand_qkv(3, S, 1, 1, D)
    o, lse = rn.attn_fwd(q, k, v, 0.5)
    oc, lsec = rs.attn_fwd(q, k, v, softmax_scale=0.5)
    for i in (0, 7, 20):
        s = 0.5 * (k[: i + 1, 0] @ q[i, 0])
        assert abs(lse[0, i] - scipy.special.logsumexp(s)) < 1e-13
        assert abs(lsec[0, i] - scipy.special.logsumexp(s)) < 1e-13
        np.testing.assert_allclose(o[i, 0], scipy.special.softmax(s) @ v[: i + 1, 0], atol=1e-13)
        np.testing.assert_allclose(oc[i, 0], scipy.special.softmax(s) @ v[: i + 1, 0], atol=1e-13)


@pytest.mark.parametrize("impl", ["numpy", "c"])
def test_fwd_closed_forms(impl):
    S, Hq, Hkv, D = 37, 4, 2, 8
    q, k, v, _ = rand_qkv(4, S, Hq, Hkv, D)
    fwd = rn.attn_fwd if impl == "numpy" else (lambda q, k, v, s=None: rs.attn_fwd(q, k, v, softmax_scale=s))
    scale = 0.3
    o, lse = fwd(q, k, v, scale)
    # first row sees one key
    for a in range(Hq):
        np.testing.assert_allclose(o[0, a], v[0, a // 2], atol=1e-15)
        assert abs(lse[a, 0] - scale * q[0, a] @ k[0, a // 2]) < 1e-14
    # zero queries: uniform weights -> prefix means, LSE = ln(i+1)
    o0, l0 = fwd(np.zeros_like(q), k, v, scale)
    pm = np.cumsum(v, axis=0) / np.arange(1, S + 1)[:, None, None]
    np.testing.assert_allclose(o0, np.repeat(pm, 2, axis=1), atol=1e-14)
    np.testing.assert_allclose(l0, np.tile(np.log(np.arange(1, S + 1)), (Hq, 1)), atol=1e-14)
    # constant values: weights sum to one
    o1, _ = fwd(q, k, np.full_like(v, 1.25), scale)
    np.testing.assert_allclose(o1, 1.25, atol=1e-14)
    # shifting every key by c moves LSE_i by scale*q_i.c and leaves O alone
    c = np.linspace(-1, 1, D)
    o2, l2 = fwd(q, k + c, v, scale)
    np.testing.assert_allclose(o2, o, atol=1e-13)
    np.testing.assert_allclose(l2 - lse, scale * np.einsum("iad,d->ai", q, c), atol=1e-13)
    # grouped-query == full attention with repeated K/V heads
    o3, l3 = fwd(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1), scale)
    np.testing.assert_allclose(o3, o, atol=1e-15)
    np.testing.assert_allclose(l3, lse, atol=1e-15)
    # causality: changing the future does not change the past
    k2, v2 = k.copy(), v.copy()
    k2[20:] += 3.0; v2[20:] -= 2.0
    o4, l4 = fwd(q, k2, v2, scale)
    assert np.array_equal(o4[:20], o[:20]) and np.array_equal(l4[:, :20], lse[:, :20])
    assert not np.allclose(o4[20:], o[20:])


# ----------------------------------------------------------- attention backward
def loss(q, k, v, do, scale):
    return float((rn.attn_fwd(q, k, v, scale)[0] * do).sum())


@pytest.mark.parametrize("impl", ["numpy", "c"])
def test_bwd_finite_differences(impl):
    S, Hq, Hkv, D = 11, 4, 2, 4
    q, k, v, do = rand_qkv(5, S, Hq, Hkv, D)
    scale = 0.6
    if impl == "numpy":
        dq, dk, dv, _ = rn.attn_bwd(q, k, v, do, scale)
    else:
        dq, dk, dv, _ = rs.attn_bwd(q, k, v, do, softmax_scale=scale)
    eps = 1e-5
    rng = np.random.default_rng(0)
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(12):
            idx = tuple(rng.integers(0, n) for n in x.shape)
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps; xm[idx] -= eps
            args_p = {"q": q, "k": k, "v": v}; args_m = dict(args_p)
            args_p[name] = xp; args_m[name] = xm
            fd = (loss(args_p["q"], args_p["k"], args_p["v"], do, scale)
                  - loss(args_m["q"], args_m["k"], args_m["v"], do, scale)) / (2 * eps)
            assert abs(fd - g[idx]) < 1e-7, (name, idx, fd, g[idx])


@pytest.mark.parametrize("impl", ["numpy", "c"])
def test_bwd_invariants(impl):
    S, Hq, Hkv, D = 29, 6, 2, 8
    G = Hq // Hkv
    q, k, v, do = rand_qkv(6, S, Hq, Hkv, D)
    scale = 0.4
    bwd = (lambda *a: rn.attn_bwd(*a, scale)) if impl == "numpy" else (lambda *a: rs.attn_bwd(*a, softmax_scale=scale))
    dq, dk, dv, delta = bwd(q, k, v, do)
    # softmax weights sum to one => dV summed over keys = dO summed over rows, per group
    np.testing.assert_allclose(dv.sum(axis=0), do.reshape(S, Hkv, G, D).sum(axis=(0, 2)), atol=1e-12)
    # last key is seen by the last row only
    o, lse = rn.attn_fwd(q, k, v, scale)
    for g in range(Hkv):
        want = np.zeros(D)
        for a in range(g * G, (g + 1) * G):
            p_last = math.exp(scale * q[S - 1, a] @ k[S - 1, g] - lse[a, S - 1])
            want += p_last * do[S - 1, a]
        np.testing.assert_allclose(dv[S - 1, g], want, atol=1e-13)
    # O depends on q and k only through q.k: scaling q by t and k by 1/t is a no-op
    assert abs((q * dq).sum() - (k * dk).sum()) < 1e-11
    # shifting every key by a common vector changes no weight: sum_j dK_j = 0
    np.testing.assert_allclose(dk.sum(axis=0), 0, atol=1e-12)
    # first row has a single key with weight 1: dQ_0 = 0
    np.testing.assert_allclose(dq[0], 0, atol=1e-14)
    # Delta
    np.testing.assert_allclose(delta, np.einsum("iad,iad->ai", do, o), atol=1e-13)
    # grouped gradient = sum over the group of the full-attention gradients
    dq_m, dk_m, dv_m, _ = bwd(q, np.repeat(k, G, axis=1), np.repeat(v, G, axis=1), do)
    np.testing.assert_allclose(dq_m, dq, atol=1e-14)
    np.testing.assert_allclose(dk_m.reshape(S, Hkv, G, D).sum(axis=2), dk, atol=1e-13)
    np.testing.assert_allclose(dv_m.reshape(S, Hkv, G, D).sum(axis=2), dv, atol=1e-13)


def test_c_oracle_matches_numpy_medium():
    S, Hq, Hkv, D = 300, 4, 2, 64
    q, k, v, do = rand_qkv(7, S, Hq, Hkv, D)
    o_n, l_n = rn.attn_fwd(q, k, v)
    dq_n, dk_n, dv_n, de_n = rn.attn_bwd(q, k, v, do)
    o_c, l_c = rs.attn_fwd(q, k, v)
    dq_c, dk_c, dv_c, de_c = rs.attn_bwd(q, k, v, do)
    for a, b in ((o_c, o_n), (l_c, l_n), (dq_c, dq_n), (dk_c, dk_n), (dv_c, dv_n), (de_c, de_n)):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-11)


def test_c_oracle_sampled_rows_and_sparse_dO():
    """Sampled rows equal the same rows of the full result; with dO non-zero on
    a row subset only, the column pass over that subset is the whole dK/dV
    (rows with dO_i = 0 contribute nothing: dP_ij = 0 and Delta_i = 0)."""
    S, Hq, Hkv, D = 200, 4, 1, 16
    q, k, v, do = rand_qkv(8, S, Hq, Hkv, D)
    rows = np.array([0, 3, 64, 65, 127, 199])
    r = rs.attn_rows(q, k, v, rows, do)
    o, lse = rn.attn_fwd(q, k, v)
    dq, _, _, delta = rn.attn_bwd(q, k, v, do)
    np.testing.assert_allclose(r["O"], o[rows], atol=1e-12)
    np.testing.assert_allclose(r["lse"], lse[:, rows], atol=1e-12)
    np.testing.assert_allclose(r["delta"], delta[:, rows], atol=1e-12)
    np.testing.assert_allclose(r["dQ"], dq[rows], atol=1e-12)
    do_sparse = np.zeros_like(do)
    do_sparse[rows] = do[rows]
    dq_s, dk_s, dv_s, _ = rn.attn_bwd(q, k, v, do_sparse)
    r2 = rs.attn_rows(q, k, v, rows, do_sparse)
    dk_c, dv_c = rs.attn_cols(q, k, v, do_sparse, rows, r2["lse"], r2["delta"], np.arange(S))
    np.testing.assert_allclose(dk_c, dk_s, atol=1e-12)
    np.testing.assert_allclose(dv_c, dv_s, atol=1e-12)
    assert np.abs(np.delete(dq_s, rows, axis=0)).max() == 0.0
    np.testing.assert_allclose(r2["dQ"], dq_s[rows], atol=1e-12)


# ----------------------------------------------------------------------- varlen
def test_varlen_equals_per_document_and_isolates_documents():
    Hq, Hkv, D = 4, 2, 8
    lengths = [5, 0, 17, 1, 9]
    cu = synth.cu_seqlens_from_lengths(lengths)
    T = int(cu[-1])
    q, k, v, do = rand_qkv(9, T, Hq, Hkv, D)
    o_c, l_c = rs.attn_fwd(q, k, v, cu_seqlens=cu)
    dq_c, dk_c, dv_c, _ = rs.attn_bwd(q, k, v, do, cu_seqlens=cu)
    o_n, l_n = rn.attn_varlen_fwd(q, k, v, cu)
    dq_n, dk_n, dv_n, _ = rn.attn_varlen_bwd(q, k, v, do, cu)
    for a, b in ((o_c, o_n), (l_c, l_n), (dq_c, dq_n), (dk_c, dk_n), (dv_c, dv_n)):
        np.testing.assert_allclose(a, b, atol=1e-12)
    # against the torch route, one document at a time
    for t in range(len(lengths)):
        a, b = cu[t], cu[t + 1]
        if b == a:
            continue
        o_t, l_t, dq_t, dk_t, dv_t = torch_reference(q[a:b], k[a:b], v[a:b], do[a:b], 1 / math.sqrt(D), 2)
        np.testing.assert_allclose(o_c[a:b], o_t, atol=1e-12)
        np.testing.assert_allclose(dk_c[a:b], dk_t, atol=1e-12)
        np.testing.assert_allclose(dv_c[a:b], dv_t, atol=1e-12)
        np.testing.assert_allclose(dq_c[a:b], dq_t, atol=1e-12)
    # poisoning one document leaves the others bit-identical
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    k2[5:22] = 1e30; v2[5:22] = -1e30; q2[5:22] = 7.0
    o_p, l_p = rs.attn_fwd(q2, k2, v2, cu_seqlens=cu)
    keep = np.r_[0:5, 22:T]
    assert np.array_equal(o_p[keep], o_c[keep]) and np.array_equal(l_p[:, keep], l_c[:, keep])
    # one document == dense
    o_d, l_d = rs.attn_fwd(q, k, v)
    o_1, l_1 = rs.attn_fwd(q, k, v, cu_seqlens=[0, T])
    assert np.array_equal(o_d, o_1) and np.array_equal(l_d, l_1)
    np.testing.assert_allclose(o_d, rn.attn_fwd(q, k, v)[0], atol=1e-12)


def test_varlen_document_permutation():
    Hq, Hkv, D = 2, 1, 4
    lengths = [4, 7, 3]
    cu = synth.cu_seqlens_from_lengths(lengths)
    q, k, v, _ = rand_qkv(10, 14, Hq, Hkv, D)
    o, _ = rs.attn_fwd(q, k, v, cu_seqlens=cu)
    order = [2, 0, 1]
    idx = np.concatenate([np.arange(cu[t], cu[t + 1]) for t in order])
    cu2 = synth.cu_seqlens_from_lengths([lengths[t] for t in order])
    o2, _ = rs.attn_fwd(q[idx], k[idx], v[idx], cu_seqlens=cu2)
    assert np.array_equal(o2, o[idx])


# ------------------------------------------------- Ulysses data flow == unsharded
def test_simulated_sequence_parallel_equals_single_device():
    """P simulated ranks: pack -> exchange -> attention on own heads over the
    whole sequence -> exchange back -> unpack, equals attention over all heads
    on one device (the rewrite must preserve semantics: Section 3.1)."""
    P, S, Hq, Hkv, D = 2, 24, 8, 4, 4
    S_l = S // P
    q, k, v, _ = rand_qkv(11, S, Hq, Hkv, D)
    o_ref, _ = rn.attn_fwd(q, k, v)

    def to_head_shards(x):
        H = x.shape[1]
        sends = []
        for r in range(P):
            packed = rn.pack_seq_to_head(x[r * S_l:(r + 1) * S_l], P)
            sends.append([packed[p * S_l:(p + 1) * S_l] for p in range(P)])
        return [np.concatenate(c, axis=0) for c in simulate_all_to_all(sends)]

    qs, ks, vs = to_head_shards(q), to_head_shards(k), to_head_shards(v)
    os_ = [rn.attn_fwd(qs[p], ks[p], vs[p])[0] for p in range(P)]
    sends_back = [[os_[p][r * S_l:(r + 1) * S_l] for r in range(P)] for p in range(P)]
    recv = simulate_all_to_all(sends_back)
    for r in range(P):
        o_local = rn.unpack_head_to_seq(np.concatenate(recv[r], axis=0), P)
        assert np.array_equal(o_local, o_ref[r * S_l:(r + 1) * S_l])


def test_flop_formula_matches_paper_count():
    """Causal forward with both contractions counted over the unmasked pairs is
    the paper's 2*b*h*s^2*d up to (s+1)/s (Section 3.2 FLOP model)."""
    b, h, s, d = 1, 4, 131072, 128
    pairs = s * (s + 1) // 2
    ours = 4 * d * h * pairs
    paper = 2 * b * h * s * s * d
    assert abs(ours / paper - (s + 1) / s) < 1e-12
