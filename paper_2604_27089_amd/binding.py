"""ctypes binding of libsp_hotpath.so: argument marshalling only.

Function names and argument order mirror include/sp_hotpath.h.  Tensors are
torch CUDA(HIP) tensors used purely as device memory; the stream is torch's
current stream unless one is given.  There is no fallback: a missing library
raises ImportError at first use, and a non-zero status raises SpError.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SP_HOTPATH_LIB points at another build of the same library (e.g. an experimental variant).
LIB_PATH = os.environ.get("SP_HOTPATH_LIB") or os.path.join(_HERE, "libsp_hotpath.so")

SP_OK, SP_ERR_NULL, SP_ERR_SHAPE, SP_ERR_UNSUPPORTED, SP_ERR_WORKSPACE, SP_ERR_ALIGN, SP_ERR_LAUNCH = range(7)

EXPORTS = (
    "sp_status_str", "sp_abi_version", "sp_pack_seq_to_head", "sp_unpack_head_to_seq", "sp_attn_fwd",
    "sp_attn_bwd_workspace_bytes", "sp_attn_varlen_fwd_workspace_bytes", "sp_attn_bwd", "sp_attn_bwd_stages",
    "sp_attn_varlen_fwd", "sp_attn_varlen_bwd", "sp_attn_varlen_fwd_static", "sp_varlen_check_cu_seqlens", "sp_attn_fwd_seqlayout", "sp_attn_bwd_seqlayout",
    "sp_attn_block_fwd", "sp_attn_merge", "sp_attn_block_bwd_workspace_bytes", "sp_attn_block_bwd",
    "sp_rmsnorm_bwd_workspace_bytes", "sp_rmsnorm_fwd", "sp_rmsnorm_bwd", "sp_rope", "sp_swiglu_fwd", "sp_swiglu_bwd",
)


class SpError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_str(code)}")


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library (once).  Fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    _lib = open_library(LIB_PATH)
    return _lib


def open_library(path: str) -> ctypes.CDLL:
    """Load a build of the library and declare its entry points (tests compare two builds through this)."""
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2604_27089_amd.build` "
                          "(there is no CPU or PyTorch fallback)")
    L = ctypes.CDLL(path)
    c = ctypes
    vp, i64, i32, f32, sz = c.c_void_p, c.c_int64, c.c_int32, c.c_float, c.c_size_t
    L.sp_status_str.restype = c.c_char_p; L.sp_status_str.argtypes = [c.c_int]
    L.sp_abi_version.restype = i32; L.sp_abi_version.argtypes = []
    for name in ("sp_pack_seq_to_head", "sp_unpack_head_to_seq"):
        f = getattr(L, name); f.restype = c.c_int
        f.argtypes = [vp, vp, i64, i64, i64, i64, i32, i32, vp]
    L.sp_attn_fwd.restype = c.c_int
    L.sp_attn_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, i32, f32, vp]
    L.sp_attn_bwd_workspace_bytes.restype = sz
    L.sp_attn_bwd_workspace_bytes.argtypes = [i64, i64, i32, i32, i32, i32]
    L.sp_attn_varlen_fwd_workspace_bytes.restype = sz
    L.sp_attn_varlen_fwd_workspace_bytes.argtypes = [i64, i32, i32, i32, i32]
    L.sp_attn_bwd.restype = c.c_int
    L.sp_attn_bwd.argtypes = [vp] * 10 + [sz, i64, i64, i32, i32, i32, f32, vp]
    L.sp_attn_bwd_stages.restype = c.c_int
    L.sp_attn_bwd_stages.argtypes = [vp] * 10 + [sz, i64, i64, i32, i32, i32, f32, i32, vp]
    L.sp_attn_fwd_seqlayout.restype = c.c_int
    L.sp_attn_fwd_seqlayout.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, i32, i32, f32, vp]
    L.sp_attn_bwd_seqlayout.restype = c.c_int
    L.sp_attn_bwd_seqlayout.argtypes = [vp] * 10 + [sz, i64, i64, i32, i32, i32, i32, f32, vp]
    L.sp_attn_block_fwd.restype = c.c_int
    L.sp_attn_block_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, i64, f32, vp]
    L.sp_attn_merge.restype = c.c_int
    L.sp_attn_merge.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, i32, vp]
    L.sp_attn_block_bwd_workspace_bytes.restype = sz
    L.sp_attn_block_bwd_workspace_bytes.argtypes = [i64, i64, i64, i32, i32, i32]
    L.sp_attn_block_bwd.restype = c.c_int
    L.sp_attn_block_bwd.argtypes = [vp] * 10 + [sz, i64, i64, i64, i32, i32, i32, i64, f32, i32, vp]
    L.sp_attn_varlen_fwd.restype = c.c_int
    L.sp_attn_varlen_fwd.argtypes = [vp] * 6 + [i32, i32, i64, i32, i32, i32, f32, vp, sz, vp]
    L.sp_attn_varlen_fwd_static.restype = c.c_int
    L.sp_attn_varlen_fwd_static.argtypes = [vp] * 6 + [i32, i32, i64, i32, i32, i32, f32, vp]
    L.sp_varlen_check_cu_seqlens.restype = c.c_int
    L.sp_varlen_check_cu_seqlens.argtypes = [vp, i32, i64, vp, vp]
    L.sp_attn_varlen_bwd.restype = c.c_int
    L.sp_attn_varlen_bwd.argtypes = [vp] * 10 + [i32, i32, i64, i32, i32, i32, f32, vp, sz, vp]
    L.sp_rmsnorm_bwd_workspace_bytes.restype = sz
    L.sp_rmsnorm_bwd_workspace_bytes.argtypes = [i64, i32]
    L.sp_rmsnorm_fwd.restype = c.c_int
    L.sp_rmsnorm_fwd.argtypes = [vp, vp, vp, vp, i64, i32, f32, vp]
    L.sp_rmsnorm_bwd.restype = c.c_int
    L.sp_rmsnorm_bwd.argtypes = [vp] * 7 + [sz, i64, i32, vp]
    L.sp_rope.restype = c.c_int
    L.sp_rope.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, vp]
    L.sp_swiglu_fwd.restype = c.c_int
    L.sp_swiglu_fwd.argtypes = [vp, vp, vp, i64, vp]
    L.sp_swiglu_bwd.restype = c.c_int
    L.sp_swiglu_bwd.argtypes = [vp] * 5 + [i64, vp]
    return L


def status_str(code: int) -> str:
    return lib().sp_status_str(int(code)).decode()


def _check(code: int, where: str):
    if code != SP_OK:
        raise SpError(code, where)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _expect(t: torch.Tensor, shape, dtype, name: str):
    """The C ABI sees pointers only: extents and element types are checked here, before any launch."""
    if tuple(t.shape) != tuple(int(x) for x in shape) or t.dtype != dtype:
        raise ValueError(f"{name}: expected {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")


def _new(stream, shape, dtype, device) -> torch.Tensor:
    """A tensor allocated by a wrapper.  torch's allocator ties a block to the stream that was current when it
    was allocated; when the kernels go to another stream the block is marked as in use there, so that it is
    not handed out again while they are still queued."""
    t = torch.empty(tuple(int(x) for x in shape), dtype=dtype, device=device)
    if stream is not None:
        t.record_stream(stream)
    return t


def _attn_shapes(q, k, v, lse_shape, kv_like_q_dims: int, o=None, lse=None, do=None, dq=None, dk=None, dv=None):
    """bf16 everywhere, k/v agree, the leading `kv_like_q_dims` extents of k equal q's, the head dim agrees."""
    bf = torch.bfloat16
    _expect(q, q.shape, bf, "q")
    kshape = tuple(q.shape[:kv_like_q_dims]) + tuple(k.shape[kv_like_q_dims:-1]) + (q.shape[-1],)
    _expect(k, kshape, bf, "k")
    _expect(v, k.shape, bf, "v")
    for t, like, name in ((o, q, "o"), (do, q, "dO"), (dq, q, "dq"), (dk, k, "dk"), (dv, k, "dv")):
        if t is not None:
            _expect(t, like.shape, bf, name)
    if lse is not None:
        _expect(lse, lse_shape, torch.float32, "lse")


# --------------------------------------------------------------------------- re-layout
def sp_pack_seq_to_head(x: torch.Tensor, P: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """x [B, S_l, H, D] -> out [B, P*S_l, H/P, D]."""
    B, S_l, H, D = x.shape
    shape = (B, P * S_l, H // P if P > 0 else H, D)
    if out is None:
        out = _new(stream, shape, x.dtype, x.device)
    elif P > 0 and H % P == 0:
        _expect(out, shape, x.dtype, "out")
    _check(lib().sp_pack_seq_to_head(_ptr(x), _ptr(out), B, S_l, H, D, P, x.element_size(), _stream(stream)),
           "sp_pack_seq_to_head")
    return out


def sp_unpack_head_to_seq(y: torch.Tensor, P: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """y [B, P*S_l, h, D] -> out [B, S_l, P*h, D]."""
    B, PS, h, D = y.shape
    if P <= 0 or PS % P != 0:
        raise ValueError(f"y has {PS} rows, not a multiple of P = {P}")
    S_l, H = PS // P, h * P
    if out is None:
        out = _new(stream, (B, S_l, H, D), y.dtype, y.device)
    else:
        _expect(out, (B, S_l, H, D), y.dtype, "out")
    _check(lib().sp_unpack_head_to_seq(_ptr(y), _ptr(out), B, S_l, H, D, P, y.element_size(), _stream(stream)),
           "sp_unpack_head_to_seq")
    return out


# --------------------------------------------------------------------------- attention
def sp_attn_fwd(q, k, v, softmax_scale: float = 0.0, o=None, lse=None, stream=None):
    """q [B,S,Hq,D], k,v [B,S,Hkv,D] bf16 -> (o [B,S,Hq,D] bf16, lse [B,Hq,S] fp32)."""
    B, S, Hq, D = q.shape
    Hkv = k.shape[2]
    _attn_shapes(q, k, v, (B, Hq, S), 2, o=o, lse=lse)
    o = _new(stream, q.shape, q.dtype, q.device) if o is None else o
    lse = _new(stream, (B, Hq, S), torch.float32, q.device) if lse is None else lse
    _check(lib().sp_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, S, Hq, Hkv, D,
                             float(softmax_scale), _stream(stream)), "sp_attn_fwd")
    return o, lse


def sp_attn_bwd_workspace_bytes(B, S_or_T, Hq, Hkv, D, n_docs=0) -> int:
    return int(lib().sp_attn_bwd_workspace_bytes(B, S_or_T, Hq, Hkv, D, n_docs))


def sp_attn_varlen_fwd_workspace_bytes(T, Hq, Hkv, D, n_docs) -> int:
    return int(lib().sp_attn_varlen_fwd_workspace_bytes(T, Hq, Hkv, D, n_docs))


def _workspace(nbytes: int, device, stream=None) -> torch.Tensor:
    return _new(stream, (max(int(nbytes), 256),), torch.uint8, device)


def _grads(stream, q, k, v, dq, dk, dv):
    return (_new(stream, q.shape, q.dtype, q.device) if dq is None else dq,
            _new(stream, k.shape, k.dtype, k.device) if dk is None else dk,
            _new(stream, v.shape, v.dtype, v.device) if dv is None else dv)


def sp_attn_bwd(q, k, v, o, lse, do, softmax_scale: float = 0.0, dq=None, dk=None, dv=None,
                workspace=None, stream=None):
    """Returns (dq, dk, dv), bf16, shaped like q, k, v."""
    B, S, Hq, D = q.shape
    Hkv = k.shape[2]
    _attn_shapes(q, k, v, (B, Hq, S), 2, o=o, lse=lse, do=do, dq=dq, dk=dk, dv=dv)
    dq, dk, dv = _grads(stream, q, k, v, dq, dk, dv)
    if workspace is None:
        workspace = _workspace(sp_attn_bwd_workspace_bytes(B, S, Hq, Hkv, D, 0), q.device, stream)
    _check(lib().sp_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(do), _ptr(dq), _ptr(dk),
                             _ptr(dv), _ptr(workspace), workspace.numel() * workspace.element_size(), B, S, Hq,
                             Hkv, D, float(softmax_scale), _stream(stream)), "sp_attn_bwd")
    return dq, dk, dv


SP_BWD_STAGE_DELTA, SP_BWD_STAGE_DKDV, SP_BWD_STAGE_DQ, SP_BWD_STAGE_ALL = 1, 2, 4, 7


def sp_attn_bwd_stages(q, k, v, o, lse, do, dq, dk, dv, workspace, stages: int, softmax_scale: float = 0.0,
                       stream=None):
    """One or more stages of the backward (bit mask of SP_BWD_STAGE_*); buffers are the caller's."""
    B, S, Hq, D = q.shape
    Hkv = k.shape[2]
    _attn_shapes(q, k, v, (B, Hq, S), 2, o=o, lse=lse, do=do, dq=dq, dk=dk, dv=dv)
    _check(lib().sp_attn_bwd_stages(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(do), _ptr(dq),
                                    _ptr(dk), _ptr(dv), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), B, S, Hq, Hkv, D,
                                    float(softmax_scale), int(stages), _stream(stream)), "sp_attn_bwd_stages")
    return dq, dk, dv


def _seq_heads(q, k, P: int):
    if P <= 0 or q.shape[2] % P != 0 or k.shape[2] % P != 0:
        raise ValueError(f"head counts {q.shape[2]} / {k.shape[2]} are not multiples of P = {P}")
    return q.shape[2] // P, k.shape[2] // P


def sp_attn_fwd_seqlayout(q, k, v, P: int, softmax_scale: float = 0.0, o=None, lse=None, stream=None):
    """Sequence-side tensors q [B,S_l,P*Hq,D], k,v [B,S_l,P*Hkv,D] -> (o [B,S_l,P*Hq,D], lse [B,Hq,P*S_l])."""
    B, S_l, _, D = q.shape
    Hq, Hkv = _seq_heads(q, k, P)
    _attn_shapes(q, k, v, (B, Hq, P * S_l), 2, o=o, lse=lse)
    o = _new(stream, q.shape, q.dtype, q.device) if o is None else o
    lse = _new(stream, (B, Hq, P * S_l), torch.float32, q.device) if lse is None else lse
    _check(lib().sp_attn_fwd_seqlayout(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, S_l, Hq, Hkv, D, P,
                                       float(softmax_scale), _stream(stream)), "sp_attn_fwd_seqlayout")
    return o, lse


def sp_attn_bwd_seqlayout(q, k, v, o, lse, do, P: int, softmax_scale: float = 0.0, dq=None, dk=None, dv=None,
                          workspace=None, stream=None):
    """Backward on sequence-side tensors; returns (dq, dk, dv) shaped like q, k, v."""
    B, S_l, _, D = q.shape
    Hq, Hkv = _seq_heads(q, k, P)
    _attn_shapes(q, k, v, (B, Hq, P * S_l), 2, o=o, lse=lse, do=do, dq=dq, dk=dk, dv=dv)
    dq, dk, dv = _grads(stream, q, k, v, dq, dk, dv)
    if workspace is None:
        workspace = _workspace(sp_attn_bwd_workspace_bytes(B, P * S_l, Hq, Hkv, D, 0), q.device, stream)
    _check(lib().sp_attn_bwd_seqlayout(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(do), _ptr(dq),
                                       _ptr(dk), _ptr(dv), _ptr(workspace),
                                       workspace.numel() * workspace.element_size(), B, S_l, Hq, Hkv,
                                       D, P, float(softmax_scale), _stream(stream)), "sp_attn_bwd_seqlayout")
    return dq, dk, dv


def sp_attn_block_fwd(q, k, v, causal_offset: int, softmax_scale: float = 0.0, o=None, lse=None, stream=None):
    """q [B,Sq,Hq,D], k,v [B,Skv,Hkv,D]; row i sees keys j <= i + causal_offset -> (o, lse [B,Hq,Sq])."""
    B, Sq, Hq, D = q.shape
    Skv, Hkv = k.shape[1], k.shape[2]
    _attn_shapes(q, k, v, (B, Hq, Sq), 1, o=o, lse=lse)
    o = _new(stream, q.shape, q.dtype, q.device) if o is None else o
    lse = _new(stream, (B, Hq, Sq), torch.float32, q.device) if lse is None else lse
    _check(lib().sp_attn_block_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Sq, Skv, Hq, Hkv, D,
                                   int(causal_offset), float(softmax_scale), _stream(stream)), "sp_attn_block_fwd")
    return o, lse


def sp_attn_merge(o_acc, lse_acc, o_blk, lse_blk, o_out=None, stream=None):
    """Folds (o_blk bf16, lse_blk) into the running (o_acc fp32 [B,S,Hq,D], lse_acc fp32 [B,Hq,S]) in place;
    also writes the merged O as bf16 into o_out if given."""
    B, S, Hq, D = o_acc.shape
    _expect(o_acc, (B, S, Hq, D), torch.float32, "o_acc")
    _expect(lse_acc, (B, Hq, S), torch.float32, "lse_acc")
    _expect(o_blk, (B, S, Hq, D), torch.bfloat16, "o_blk")
    _expect(lse_blk, (B, Hq, S), torch.float32, "lse_blk")
    if o_out is not None:
        _expect(o_out, (B, S, Hq, D), torch.bfloat16, "o_out")
    _check(lib().sp_attn_merge(_ptr(o_acc), _ptr(lse_acc), _ptr(o_blk), _ptr(lse_blk), _ptr(o_out), B, S, Hq, D,
                               _stream(stream)), "sp_attn_merge")
    return o_acc, lse_acc


def sp_attn_block_bwd_workspace_bytes(B, Sq, Skv, Hq, Hkv, D) -> int:
    return int(lib().sp_attn_block_bwd_workspace_bytes(B, Sq, Skv, Hq, Hkv, D))


def sp_attn_block_bwd(q, k, v, o, lse, do, causal_offset: int, softmax_scale: float = 0.0, dq=None, dk=None,
                      dv=None, workspace=None, stages: int = SP_BWD_STAGE_ALL, stream=None):
    """This block pair's shares (dq, dk, dv), from the final o, lse of the query rows."""
    B, Sq, Hq, D = q.shape
    Skv, Hkv = k.shape[1], k.shape[2]
    _attn_shapes(q, k, v, (B, Hq, Sq), 1, o=o, lse=lse, do=do, dq=dq, dk=dk, dv=dv)
    dq, dk, dv = _grads(stream, q, k, v, dq, dk, dv)
    if workspace is None:
        workspace = _workspace(sp_attn_block_bwd_workspace_bytes(B, Sq, Skv, Hq, Hkv, D), q.device, stream)
    _check(lib().sp_attn_block_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(do), _ptr(dq), _ptr(dk),
                                   _ptr(dv), _ptr(workspace), workspace.numel() * workspace.element_size(), B, Sq,
                                   Skv, Hq, Hkv, D, int(causal_offset), float(softmax_scale), int(stages),
                                   _stream(stream)),
           "sp_attn_block_bwd")
    return dq, dk, dv


def _docs(cu_seqlens) -> int:
    if cu_seqlens.dtype != torch.int32 or cu_seqlens.dim() != 1 or cu_seqlens.numel() < 1:
        raise ValueError(f"cu_seqlens: expected a device int32 vector of n_docs + 1 entries, got "
                         f"{cu_seqlens.dtype} {tuple(cu_seqlens.shape)}")
    return cu_seqlens.numel() - 1


def sp_attn_varlen_fwd(q, k, v, cu_seqlens, max_seqlen: int = 0, softmax_scale: float = 0.0, o=None,
                       lse=None, workspace=None, stream=None):
    """q [T,Hq,D], k,v [T,Hkv,D]; cu_seqlens device int32 [n_docs+1] -> (o, lse [Hq,T])."""
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    n_docs = _docs(cu_seqlens)
    _attn_shapes(q, k, v, (Hq, T), 1, o=o, lse=lse)
    o = _new(stream, q.shape, q.dtype, q.device) if o is None else o
    lse = _new(stream, (Hq, T), torch.float32, q.device) if lse is None else lse
    if workspace is None:
        workspace = _workspace(sp_attn_varlen_fwd_workspace_bytes(T, Hq, Hkv, D, n_docs), q.device, stream)
    _check(lib().sp_attn_varlen_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(cu_seqlens), n_docs,
                                    int(max_seqlen), T, Hq, Hkv, D, float(softmax_scale), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)),
           "sp_attn_varlen_fwd")
    return o, lse


def sp_attn_varlen_fwd_static(q, k, v, cu_seqlens, o, lse, max_seqlen: int = 0, softmax_scale: float = 0.0, stream=None):
    """sp_attn_varlen_fwd on the library's own static scratch: allocates nothing, so o and lse are the caller's."""
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    n_docs = _docs(cu_seqlens)
    _attn_shapes(q, k, v, (Hq, T), 1, o=o, lse=lse)
    _check(lib().sp_attn_varlen_fwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(cu_seqlens), n_docs,
                                           int(max_seqlen), T, Hq, Hkv, D, float(softmax_scale), _stream(stream)),
           "sp_attn_varlen_fwd_static")
    return o, lse


def sp_varlen_check_cu_seqlens(cu_seqlens, T: int, flag=None, stream=None):
    """Debug aid: returns a device int32 tensor holding 0 if cu_seqlens is well formed for T rows, else a bit
    mask (1: cu[0] != 0, 2: decreasing somewhere, 4: cu[-1] != T).  Does not synchronise."""
    n_docs = _docs(cu_seqlens)
    flag = _new(stream, (1,), torch.int32, cu_seqlens.device) if flag is None else flag
    _expect(flag, (1,), torch.int32, "flag")
    _check(lib().sp_varlen_check_cu_seqlens(_ptr(cu_seqlens), n_docs, int(T), _ptr(flag), _stream(stream)),
           "sp_varlen_check_cu_seqlens")
    return flag


def sp_attn_varlen_bwd(q, k, v, o, lse, do, cu_seqlens, max_seqlen: int = 0, softmax_scale: float = 0.0,
                       dq=None, dk=None, dv=None, workspace=None, stream=None):
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    n_docs = _docs(cu_seqlens)
    _attn_shapes(q, k, v, (Hq, T), 1, o=o, lse=lse, do=do, dq=dq, dk=dk, dv=dv)
    dq, dk, dv = _grads(stream, q, k, v, dq, dk, dv)
    if workspace is None:
        workspace = _workspace(sp_attn_bwd_workspace_bytes(1, T, Hq, Hkv, D, n_docs), q.device, stream)
    _check(lib().sp_attn_varlen_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _ptr(do), _ptr(dq),
                                    _ptr(dk), _ptr(dv), _ptr(cu_seqlens), n_docs, int(max_seqlen), T, Hq,
                                    Hkv, D, float(softmax_scale), _ptr(workspace),
                                    workspace.numel() * workspace.element_size(), _stream(stream)),
           "sp_attn_varlen_bwd")
    return dq, dk, dv


# --------------------------------------------------------------------------- pointwise operators
def sp_rmsnorm_fwd(x, w, eps: float, y=None, rstd=None, stream=None):
    """x [T, C] bf16, w [C] bf16 -> (y [T, C] bf16, rstd [T] fp32)."""
    T, C = x.shape
    _expect(x, (T, C), torch.bfloat16, "x"); _expect(w, (C,), torch.bfloat16, "w")
    y = _new(stream, x.shape, x.dtype, x.device) if y is None else y
    rstd = _new(stream, (T,), torch.float32, x.device) if rstd is None else rstd
    _check(lib().sp_rmsnorm_fwd(_ptr(x), _ptr(w), _ptr(y), _ptr(rstd), T, C, float(eps), _stream(stream)), "sp_rmsnorm_fwd")
    return y, rstd


def sp_rmsnorm_bwd_workspace_bytes(T, C) -> int:
    return int(lib().sp_rmsnorm_bwd_workspace_bytes(T, C))


def sp_rmsnorm_bwd(x, w, rstd, dy, dx=None, dw=None, workspace=None, stream=None):
    """Returns (dx [T, C], dw [C]) bf16."""
    T, C = x.shape
    _expect(x, (T, C), torch.bfloat16, "x"); _expect(w, (C,), torch.bfloat16, "w")
    _expect(dy, (T, C), torch.bfloat16, "dy"); _expect(rstd, (T,), torch.float32, "rstd")
    dx = _new(stream, x.shape, x.dtype, x.device) if dx is None else dx
    dw = _new(stream, w.shape, w.dtype, w.device) if dw is None else dw
    if workspace is None:
        workspace = _workspace(sp_rmsnorm_bwd_workspace_bytes(T, C), x.device, stream)
    _check(lib().sp_rmsnorm_bwd(_ptr(x), _ptr(w), _ptr(rstd), _ptr(dy), _ptr(dx), _ptr(dw), _ptr(workspace),
                                workspace.numel() * workspace.element_size(), T, C, _stream(stream)), "sp_rmsnorm_bwd")
    return dx, dw


def sp_rope(x, cos_table, sin_table, conjugate: bool = False, out=None, stream=None):
    """x [T, H, D] bf16, cos/sin tables [T, D/2] fp32 -> rotated tensor (out may be x)."""
    T, H, D = x.shape
    _expect(x, (T, H, D), torch.bfloat16, "x")
    _expect(cos_table, (T, D // 2), torch.float32, "cos_table"); _expect(sin_table, (T, D // 2), torch.float32, "sin_table")
    out = _new(stream, x.shape, x.dtype, x.device) if out is None else out
    _check(lib().sp_rope(_ptr(x), _ptr(cos_table), _ptr(sin_table), _ptr(out), T, H, D, int(bool(conjugate)),
                         _stream(stream)), "sp_rope")
    return out


def sp_swiglu_fwd(g, u, y=None, stream=None):
    _expect(g, g.shape, torch.bfloat16, "g"); _expect(u, g.shape, torch.bfloat16, "u")
    y = _new(stream, g.shape, g.dtype, g.device) if y is None else y
    _check(lib().sp_swiglu_fwd(_ptr(g), _ptr(u), _ptr(y), g.numel(), _stream(stream)), "sp_swiglu_fwd")
    return y


def sp_swiglu_bwd(g, u, dy, dg=None, du=None, stream=None):
    _expect(g, g.shape, torch.bfloat16, "g"); _expect(u, g.shape, torch.bfloat16, "u"); _expect(dy, g.shape, torch.bfloat16, "dy")
    dg = _new(stream, g.shape, g.dtype, g.device) if dg is None else dg
    du = _new(stream, u.shape, u.dtype, u.device) if du is None else du
    _check(lib().sp_swiglu_bwd(_ptr(g), _ptr(u), _ptr(dy), _ptr(dg), _ptr(du), g.numel(), _stream(stream)), "sp_swiglu_bwd")
    return dg, du


def default_scale(D: int) -> float:
    return 1.0 / math.sqrt(D)
