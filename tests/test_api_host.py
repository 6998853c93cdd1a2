"""Host-side behaviour of the C-ABI library that needs no GPU: it loads, it
exports every symbol the header declares, and argument errors come back as
status codes before any launch."""
import ctypes
import os
import re

import pytest

from paper_2604_27089_amd import binding as sp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sp_hotpath.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = sp.lib()
    names = declared_symbols()
    assert len(names) >= 10
    for n in names:
        assert hasattr(L, n), f"{n} declared in the header but not exported"
    assert set(names) == set(sp.EXPORTS)
    assert L.sp_abi_version() == 4


def test_status_strings():
    for code in range(7):
        s = sp.status_str(code)
        assert s.startswith("SP_")
    assert "unknown" in sp.status_str(99)


def A(n):  # a fake but aligned, non-null address; never dereferenced on error paths
    return ctypes.c_void_p(0x1000 * n)


def test_relayout_argument_errors():
    L = sp.lib()
    f = L.sp_pack_seq_to_head
    assert f(A(1), A(2), 1, 8, 7, 64, 4, 2, None) == sp.SP_ERR_SHAPE        # H % P
    assert f(A(1), A(2), 1, 8, 8, 64, 0, 2, None) == sp.SP_ERR_SHAPE        # P <= 0
    assert f(A(1), A(2), -1, 8, 8, 64, 4, 2, None) == sp.SP_ERR_SHAPE
    assert f(A(1), A(2), 1, 8, 8, 64, 4, 1, None) == sp.SP_ERR_UNSUPPORTED  # elem size
    assert f(A(1), A(2), 1, 8, 8, 4, 4, 2, None) == sp.SP_ERR_UNSUPPORTED   # D*2 not x16
    assert f(None, A(2), 1, 8, 8, 64, 4, 2, None) == sp.SP_ERR_NULL
    assert f(ctypes.c_void_p(0x1008), A(2), 1, 8, 8, 64, 4, 2, None) == sp.SP_ERR_ALIGN
    assert f(None, None, 1, 0, 8, 64, 4, 2, None) == sp.SP_OK               # empty
    assert L.sp_unpack_head_to_seq(A(1), A(2), 1, 8, 6, 64, 4, 2, None) == sp.SP_ERR_SHAPE


def test_attention_argument_errors():
    L = sp.lib()
    f = L.sp_attn_fwd
    assert f(A(1), A(2), A(3), A(4), A(5), 1, 128, 4, 3, 128, 0.0, None) == sp.SP_ERR_SHAPE  # Hq % Hkv
    assert f(A(1), A(2), A(3), A(4), A(5), 1, 128, 4, 1, 96, 0.0, None) == sp.SP_ERR_UNSUPPORTED
    assert f(A(1), A(2), A(3), A(4), A(5), 1, 1 << 31, 4, 1, 128, 0.0, None) == sp.SP_ERR_SHAPE
    assert f(None, A(2), A(3), A(4), A(5), 1, 128, 4, 1, 128, 0.0, None) == sp.SP_ERR_NULL
    assert f(A(1), A(2), A(3), ctypes.c_void_p(0x4004), A(5), 1, 128, 4, 1, 128, 0.0, None) == sp.SP_ERR_ALIGN
    assert f(None, None, None, None, None, 1, 0, 4, 1, 128, 0.0, None) == sp.SP_OK           # empty
    need = sp.sp_attn_bwd_workspace_bytes(1, 1024, 4, 1, 128, 0)
    assert need >= 4 * 1024 * 4
    assert sp.sp_attn_bwd_workspace_bytes(1, 1024, 4, 3, 128, 0) == 0
    assert sp.sp_attn_bwd_workspace_bytes(1, 1024, 4, 1, 128, 3) >= need + 2 * 4 * 1024
    assert sp.sp_attn_varlen_fwd_workspace_bytes(1024, 4, 1, 128, 3) >= 2 * 4 * 1024
    g = L.sp_attn_bwd
    args = [A(i) for i in range(1, 11)]
    assert g(*args, need - 1, 1, 1024, 4, 1, 128, 0.0, None) == sp.SP_ERR_WORKSPACE
    assert g(*args[:9], None, need, 1, 1024, 4, 1, 128, 0.0, None) == sp.SP_ERR_NULL
    vf = L.sp_attn_varlen_fwd
    assert vf(A(1), A(2), A(3), A(4), A(5), A(6), 0, 0, 1024, 4, 1, 128, 0.0, A(7), 1 << 20, None) == sp.SP_ERR_SHAPE
    assert vf(A(1), A(2), A(3), A(4), A(5), None, 2, 0, 1024, 4, 1, 128, 0.0, A(7), 1 << 20, None) == sp.SP_ERR_NULL
    assert vf(A(1), A(2), A(3), A(4), A(5), A(6), 2, 0, 1024, 4, 1, 128, 0.0, A(7), 16, None) == sp.SP_ERR_WORKSPACE
    vb = L.sp_attn_varlen_bwd
    assert vb(*args[:9], A(11), 2, 0, 1024, 4, 1, 128, 0.0, A(12), 16, None) == sp.SP_ERR_WORKSPACE
    # sequence-side calls: S_l must be a power of two >= 256
    sf = L.sp_attn_fwd_seqlayout
    assert sf(A(1), A(2), A(3), A(4), A(5), 1, 384, 4, 1, 128, 8, 0.0, None) == sp.SP_ERR_UNSUPPORTED
    assert sf(A(1), A(2), A(3), A(4), A(5), 1, 128, 4, 1, 128, 8, 0.0, None) == sp.SP_ERR_UNSUPPORTED
    assert sf(A(1), A(2), A(3), A(4), A(5), 1, 512, 4, 1, 128, 0, 0.0, None) == sp.SP_ERR_SHAPE
    assert sf(A(1), A(2), A(3), A(4), A(5), 1, 512, 4, 3, 128, 8, 0.0, None) == sp.SP_ERR_SHAPE
    assert sf(None, A(2), A(3), A(4), A(5), 1, 512, 4, 1, 128, 8, 0.0, None) == sp.SP_ERR_NULL
    assert sf(None, None, None, None, None, 1, 0, 4, 1, 128, 8, 0.0, None) == sp.SP_OK
    sb = L.sp_attn_bwd_seqlayout
    need8 = sp.sp_attn_bwd_workspace_bytes(1, 8 * 512, 4, 1, 128, 0)
    assert sb(*args, need8 - 1, 1, 512, 4, 1, 128, 8, 0.0, None) == sp.SP_ERR_WORKSPACE
    assert sb(*args, need8, 1, 500, 4, 1, 128, 8, 0.0, None) == sp.SP_ERR_UNSUPPORTED


def test_block_step_argument_errors():
    L = sp.lib()
    bf = L.sp_attn_block_fwd
    five = [A(i) for i in range(1, 6)]
    assert bf(*five, 1, 256, 256, 4, 1, 128, -1, 0.0, None) == sp.SP_ERR_SHAPE       # negative offset
    assert bf(*five, 1, 256, 512, 4, 1, 128, 100, 0.0, None) == sp.SP_ERR_SHAPE      # keys no row sees
    assert bf(*five, 1, 256, 512, 4, 3, 128, 511, 0.0, None) == sp.SP_ERR_SHAPE      # Hq % Hkv
    assert bf(*five, 1, 256, 512, 4, 1, 96, 511, 0.0, None) == sp.SP_ERR_UNSUPPORTED
    assert bf(*five, 1, 256, 0, 4, 1, 128, 0, 0.0, None) == sp.SP_ERR_SHAPE          # no keys at all
    assert bf(None, *five[1:], 1, 256, 512, 4, 1, 128, 511, 0.0, None) == sp.SP_ERR_NULL
    assert bf(None, None, None, None, None, 1, 0, 512, 4, 1, 128, 1 << 40, 0.0, None) == sp.SP_OK  # no rows
    need = sp.sp_attn_block_bwd_workspace_bytes(1, 1024, 2048, 4, 1, 128)
    assert need >= 4 * 1024 * 4
    assert sp.sp_attn_block_bwd_workspace_bytes(1, 1024, 2048, 4, 3, 128) == 0
    bb = L.sp_attn_block_bwd
    args = [A(i) for i in range(1, 11)]
    assert bb(*args, need - 1, 1, 1024, 2048, 4, 1, 128, 2048, 0.0, 7, None) == sp.SP_ERR_WORKSPACE
    assert bb(*args, need, 1, 1024, 2048, 4, 1, 128, 2048, 0.0, 0, None) == sp.SP_ERR_SHAPE  # no stage
    assert bb(*args, need, 1, 1024, 2048, 4, 1, 128, 512, 0.0, 7, None) == sp.SP_ERR_SHAPE
    assert bb(*args[:9], None, need, 1, 1024, 2048, 4, 1, 128, 2048, 0.0, 7, None) == sp.SP_ERR_NULL
    mg = L.sp_attn_merge
    assert mg(A(1), A(2), A(3), A(4), None, 1, 256, 4, 96, None) == sp.SP_ERR_UNSUPPORTED
    assert mg(A(1), A(2), A(3), A(4), None, 1, -1, 4, 128, None) == sp.SP_ERR_SHAPE
    assert mg(A(1), None, A(3), A(4), None, 1, 256, 4, 128, None) == sp.SP_ERR_NULL
    assert mg(A(1), A(2), A(3), A(4), ctypes.c_void_p(0x4004), 1, 256, 4, 128, None) == sp.SP_ERR_ALIGN
    assert mg(None, None, None, None, None, 1, 0, 4, 128, None) == sp.SP_OK


def test_pointwise_argument_errors():
    L = sp.lib()
    assert L.sp_rmsnorm_fwd(A(1), A(2), A(3), A(4), 4, 4100, 1e-5, None) == sp.SP_ERR_UNSUPPORTED   # C % 8
    assert L.sp_rmsnorm_fwd(A(1), A(2), A(3), A(4), 4, 16384, 1e-5, None) == sp.SP_ERR_UNSUPPORTED  # C > 8192
    assert L.sp_rmsnorm_fwd(A(1), A(2), A(3), A(4), -1, 64, 1e-5, None) == sp.SP_ERR_SHAPE
    assert L.sp_rmsnorm_fwd(A(1), A(2), A(3), A(4), 4, 64, -1.0, None) == sp.SP_ERR_SHAPE
    assert L.sp_rmsnorm_fwd(None, A(2), A(3), A(4), 4, 64, 1e-5, None) == sp.SP_ERR_NULL
    assert L.sp_rmsnorm_fwd(None, None, None, None, 0, 64, 1e-5, None) == sp.SP_OK
    need = sp.sp_rmsnorm_bwd_workspace_bytes(4096, 4096)
    assert need >= 512 * 4096 * 4 and sp.sp_rmsnorm_bwd_workspace_bytes(4096, 12) == 0
    a7 = [A(i) for i in range(1, 8)]
    assert L.sp_rmsnorm_bwd(*a7, need - 1, 4096, 4096, None) == sp.SP_ERR_WORKSPACE
    assert L.sp_rmsnorm_bwd(*a7[:6], None, need, 4096, 4096, None) == sp.SP_ERR_NULL
    assert L.sp_rope(A(1), A(2), A(3), A(4), 8, 4, 24, 0, None) == sp.SP_ERR_UNSUPPORTED  # D % 16
    assert L.sp_rope(A(1), None, A(3), A(4), 8, 4, 64, 0, None) == sp.SP_ERR_NULL
    assert L.sp_rope(A(1), A(2), A(3), ctypes.c_void_p(0x4008), 8, 4, 64, 1, None) == sp.SP_ERR_ALIGN
    assert L.sp_rope(None, None, None, None, 0, 4, 64, 0, None) == sp.SP_OK
    assert L.sp_swiglu_fwd(A(1), A(2), A(3), 12, None) == sp.SP_ERR_UNSUPPORTED           # n % 8
    assert L.sp_swiglu_fwd(A(1), A(2), None, 16, None) == sp.SP_ERR_NULL
    assert L.sp_swiglu_bwd(A(1), A(2), A(3), A(4), A(5), -8, None) == sp.SP_ERR_SHAPE
    assert L.sp_swiglu_bwd(None, None, None, None, None, 0, None) == sp.SP_OK


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(sp, "_lib", None)
    monkeypatch.setattr(sp, "LIB_PATH", "/nonexistent/libsp_hotpath.so")
    with pytest.raises(ImportError):
        sp.lib()


def test_cu_seqlens_check_argument_errors():
    f = sp.lib().sp_varlen_check_cu_seqlens
    assert f(None, 3, 100, A(2), None) == sp.SP_ERR_NULL
    assert f(A(1), 3, 100, None, None) == sp.SP_ERR_NULL
    assert f(A(1), -1, 100, A(2), None) == sp.SP_ERR_SHAPE
    assert f(A(1), 3, 1 << 31, A(2), None) == sp.SP_ERR_SHAPE
    assert f(ctypes.c_void_p(0x1002), 3, 100, A(2), None) == sp.SP_ERR_ALIGN


def test_binding_rejects_wrong_dtypes_and_shapes_before_any_launch():
    """The C ABI sees pointers only; the wrappers check element types and extents first (CPU tensors suffice:
    the checks run before any pointer is taken)."""
    import torch

    bf = torch.bfloat16
    q = torch.zeros(1, 64, 4, 128, dtype=bf); k = torch.zeros(1, 64, 1, 128, dtype=bf); v = torch.zeros_like(k)
    with pytest.raises(ValueError, match="q: expected torch.bfloat16"):
        sp.sp_attn_fwd(q.float(), k, v)
    with pytest.raises(ValueError, match="k: expected"):
        sp.sp_attn_fwd(q, k[:, :32], v[:, :32])          # fewer key rows than query rows
    with pytest.raises(ValueError, match="v: expected"):
        sp.sp_attn_fwd(q, k, torch.zeros(1, 64, 2, 128, dtype=bf))
    with pytest.raises(ValueError, match="k: expected"):
        sp.sp_attn_fwd(q, torch.zeros(1, 64, 1, 64, dtype=bf), torch.zeros(1, 64, 1, 64, dtype=bf))  # head dim
    with pytest.raises(ValueError, match="lse: expected torch.float32"):
        sp.sp_attn_fwd(q, k, v, lse=torch.zeros(1, 64, 4))
    o = torch.zeros_like(q); lse = torch.zeros(1, 4, 64)
    with pytest.raises(ValueError, match="dO: expected"):
        sp.sp_attn_bwd(q, k, v, o, lse, torch.zeros(1, 64, 4, 64, dtype=bf))
    with pytest.raises(ValueError, match="dk: expected"):
        sp.sp_attn_bwd(q, k, v, o, lse, torch.zeros_like(q), dk=torch.zeros_like(q))
    qv = q[0]; kv = k[0]
    with pytest.raises(ValueError, match="cu_seqlens"):
        sp.sp_attn_varlen_fwd(qv, kv, kv, torch.tensor([0, 64]))  # int64
    with pytest.raises(ValueError, match="lse: expected"):
        sp.sp_attn_varlen_fwd(qv, kv, kv, torch.tensor([0, 64], dtype=torch.int32), lse=torch.zeros(64, 4))
    with pytest.raises(ValueError, match="multiples of P"):
        sp.sp_attn_fwd_seqlayout(q, k, v, 3)
    with pytest.raises(ValueError, match="o_blk"):
        sp.sp_attn_merge(torch.zeros(1, 8, 2, 64), torch.zeros(1, 2, 8), torch.zeros(1, 8, 2, 64), torch.zeros(1, 2, 8))
    with pytest.raises(ValueError, match="w: expected"):
        sp.sp_rmsnorm_fwd(torch.zeros(4, 64, dtype=bf), torch.zeros(32, dtype=bf), 1e-5)
    with pytest.raises(ValueError, match="cos_table"):
        sp.sp_rope(torch.zeros(4, 2, 64, dtype=bf), torch.zeros(4, 64), torch.zeros(4, 32))
    with pytest.raises(ValueError, match="u: expected"):
        sp.sp_swiglu_fwd(torch.zeros(16, dtype=bf), torch.zeros(8, dtype=bf))
