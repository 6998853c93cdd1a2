"""The packed-document forward on the library's static scratch (for callers that cannot allocate device
memory): same bits as the workspace-taking entry point, on two calls in a row, the second smaller; a third
larger again; and the size limit is an error, not a launch.  Calls go through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2604_27089_amd import binding as sp
from paper_2604_27089_amd import synth
from gpu_util import dev_bf16

pytestmark = pytest.mark.gpu


def both(lengths, Hq, Hkv, D, seed):
    cu = synth.cu_seqlens_from_lengths(lengths)
    T = int(cu[-1])
    q, k, v, _ = synth.attn_inputs(seed, T, Hq, Hkv, D)
    qd, kd, vd = (dev_bf16(t[0]) for t in (q, k, v))
    cud = torch.from_numpy(cu).cuda()
    o_ref, lse_ref = sp.sp_attn_varlen_fwd(qd, kd, vd, cud)
    o = torch.full_like(o_ref, float("nan"))
    lse = torch.full_like(lse_ref, float("nan"))
    L = sp.lib()
    st = torch.cuda.current_stream().cuda_stream
    p = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = L.sp_attn_varlen_fwd_static(p(qd), p(kd), p(vd), p(o), p(lse), p(cud), len(lengths), 0, T, Hq, Hkv, D,
                                     0.0, ctypes.c_void_p(st))
    assert rc == sp.SP_OK, sp.status_str(rc)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), o_ref.view(torch.int16)), f"O differs for lengths {lengths}"
    assert torch.equal(lse.view(torch.int32), lse_ref.view(torch.int32)), f"LSE differs for lengths {lengths}"


def test_static_scratch_matches_workspace_entry_point_on_consecutive_calls():
    both(synth.doc_lengths(0, total=16384, mean=1024.0), 4, 1, 128, 1)   # ragged lognormal mix, 64 tiles
    both([700, 0, 333, 129], 4, 2, 64, 2)                                # smaller: stale words stay beyond it
    both(synth.doc_lengths(3, total=8192, mean=700.0, lo=16), 2, 1, 128, 3)
    both([5], 1, 1, 64, 4)


def test_static_scratch_size_limit_and_argument_errors():
    L = sp.lib()
    A = lambda n: ctypes.c_void_p(0x1000 * n)
    f = L.sp_attn_varlen_fwd_static
    big = 1 << 21  # 2M rows need 16 MiB of windows: beyond the 8 MiB scratch
    assert L.sp_attn_varlen_fwd_workspace_bytes(big, 4, 1, 128, 3) > (8 << 20)
    assert f(A(1), A(2), A(3), A(4), A(5), A(6), 3, 0, big, 4, 1, 128, 0.0, None) == sp.SP_ERR_WORKSPACE
    assert f(None, A(2), A(3), A(4), A(5), A(6), 3, 0, 1024, 4, 1, 128, 0.0, None) == sp.SP_ERR_NULL
    assert f(A(1), A(2), A(3), A(4), A(5), A(6), 0, 0, 1024, 4, 1, 128, 0.0, None) == sp.SP_ERR_SHAPE
    assert f(A(1), A(2), A(3), A(4), A(5), A(6), 3, 0, 1024, 4, 3, 128, 0.0, None) == sp.SP_ERR_SHAPE
    assert f(None, None, None, None, None, None, 0, 0, 0, 4, 1, 128, 0.0, None) == sp.SP_OK  # empty
