"""The regular build schedules its assembly MFMAs by hand: partial LDS waits counted at compile time, results
read after a counted number of instructions, no wait states.  The padded build of the same sources
(-DSP_PADDED_MFMA) waits for everything before every MFMA and spends the full result latency after it; the
arithmetic and its order are the same.  Equal bits from the two builds say the hand-counted schedule reads no
register early and no operand late, on shapes that reach every body of the pipelines (ragged tails, split key
tiles, masks, packed documents, both head dims)."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import build as spbuild
from paper_2604_27089_amd import synth
from gpu_util import dev_bf16

pytestmark = pytest.mark.gpu


def run(L, q, k, v, do, cu=None):
    """forward + backward through the C ABI of library L; returns (o, lse, dq, dk, dv)."""
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    o = torch.full_like(q, float("nan")); dq = torch.full_like(q, float("nan"))
    dk = torch.full_like(k, float("nan")); dv = torch.full_like(v, float("nan"))
    if cu is None:
        B, S, Hq, D = q.shape
        Hkv = k.shape[2]
        lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty(L.sp_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, 0), dtype=torch.uint8, device="cuda")
        assert L.sp_attn_fwd(p(q), p(k), p(v), p(o), p(lse), B, S, Hq, Hkv, D, 0.0, st) == sp.SP_OK
        assert L.sp_attn_bwd(p(q), p(k), p(v), p(o), p(lse), p(do), p(dq), p(dk), p(dv), p(ws), ws.numel(), B, S, Hq,
                             Hkv, D, 0.0, st) == sp.SP_OK
    else:
        T, Hq, D = q.shape
        Hkv = k.shape[1]
        n = cu.numel() - 1
        lse = torch.full((Hq, T), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty(L.sp_attn_bwd_workspace_bytes(1, T, Hq, Hkv, D, n), dtype=torch.uint8, device="cuda")
        assert L.sp_attn_varlen_fwd(p(q), p(k), p(v), p(o), p(lse), p(cu), n, 0, T, Hq, Hkv, D, 0.0, p(ws), ws.numel(),
                                    st) == sp.SP_OK
        assert L.sp_attn_varlen_bwd(p(q), p(k), p(v), p(o), p(lse), p(do), p(dq), p(dk), p(dv), p(cu), n, 0, T, Hq, Hkv,
                                    D, 0.0, p(ws), ws.numel(), st) == sp.SP_OK
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


def same_bits(a, b, what):
    for x, y, name in zip(a, b, ("O", "LSE", "dQ", "dK", "dV")):
        bits = torch.int32 if x.dtype == torch.float32 else torch.int16
        assert torch.equal(x.view(bits), y.view(bits)), f"{what}: {name} differs between the regular and the padded build"
        assert torch.isfinite(x.float()).all(), f"{what}: {name} not finite"


DENSE = [(1, 2100, 4, 1, 128), (2, 777, 2, 2, 64), (1, 3000, 4, 1, 64), (1, 4500, 3, 1, 128), (1, 33, 5, 5, 128)]


@pytest.mark.parametrize("B,S,Hq,Hkv,D", DENSE)
def test_padded_build_gives_the_same_bits_dense(B, S, Hq, Hkv, D):
    fast, padded = sp.lib(), sp.open_library(spbuild.LIB_PADDED)
    q, k, v, do = (dev_bf16(t) for t in synth.attn_inputs(S + D, S, Hq, Hkv, D, B))
    same_bits(run(fast, q, k, v, do), run(padded, q, k, v, do), f"B={B} S={S} {Hq}q/{Hkv}kv D={D}")


def test_padded_build_gives_the_same_bits_packed_documents():
    fast, padded = sp.lib(), sp.open_library(spbuild.LIB_PADDED)
    lengths = [130, 0, 64, 1, 700, 63, 129, 2040, 8, 30, 2, 1500]
    cu = synth.cu_seqlens_from_lengths(lengths)
    T, Hq, Hkv, D = int(cu[-1]), 4, 1, 128
    q, k, v, do = (dev_bf16(t[0]) for t in synth.attn_inputs(77, T, Hq, Hkv, D))
    cud = torch.from_numpy(cu).cuda()
    same_bits(run(fast, q, k, v, do, cud), run(padded, q, k, v, do, cud), "packed documents")
