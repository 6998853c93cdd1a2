"""ctypes front end of the streaming C oracle.  TEST INFRASTRUCTURE ONLY.

Same operator as ref_numpy, affordable at long sequence lengths and on sampled
rows/columns.  See ref_stream.c for the definition it follows.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        # REF_STREAM_LIB names another build of ref_stream.c (the sanitizer build of the test suite); it is
        # loaded as it is and never rebuilt here
        path = os.environ.get("REF_STREAM_LIB") or _build.LIB
        if path == _build.LIB and (not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC)):
            _build.build()
        _lib = ctypes.CDLL(path)
        _lib.ref_num_threads.restype = ctypes.c_int
        _lib.ref_attn_rows.restype = ctypes.c_int
        _lib.ref_attn_cols.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().ref_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _relayout(fn_name, x: np.ndarray, P: int, out_shape):
    lib = _load()
    x = np.ascontiguousarray(x)
    B, S_l, H, D = (int(t) for t in (x.shape if fn_name == "ref_pack_seq_to_head" else
                                     (x.shape[0], x.shape[1] // P, x.shape[2] * P, x.shape[3])))
    out = np.empty(out_shape, dtype=x.dtype)
    getattr(lib, fn_name)(_p(x), _p(out), ctypes.c_int64(B), ctypes.c_int64(S_l), ctypes.c_int64(H),
                          ctypes.c_int64(D), ctypes.c_int32(P), ctypes.c_int32(x.dtype.itemsize))
    return out


def pack_seq_to_head(x: np.ndarray, P: int) -> np.ndarray:
    """x [B, S_l, H, D] -> [B, P*S_l, H/P, D]."""
    B, S_l, H, D = x.shape
    assert H % P == 0
    return _relayout("ref_pack_seq_to_head", x, P, (B, P * S_l, H // P, D))


def unpack_head_to_seq(y: np.ndarray, P: int) -> np.ndarray:
    """y [B, P*S_l, h, D] -> [B, S_l, P*h, D]."""
    B, PS, h, D = y.shape
    assert PS % P == 0
    return _relayout("ref_unpack_head_to_seq", y, P, (B, PS // P, h * P, D))


def _prep(q, k, v, do, cu_seqlens, softmax_scale):
    q = np.ascontiguousarray(q, np.float64); k = np.ascontiguousarray(k, np.float64)
    v = np.ascontiguousarray(v, np.float64)
    do = None if do is None else np.ascontiguousarray(do, np.float64)
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    assert Hq % Hkv == 0 and k.shape == v.shape == (T, Hkv, D)
    if cu_seqlens is None:
        cu_seqlens = [0, T]
    cu = np.ascontiguousarray(cu_seqlens, np.int32)
    assert cu[0] == 0 and cu[-1] == T and np.all(np.diff(cu) >= 0)
    scale = float(softmax_scale) if (softmax_scale is not None and softmax_scale > 0) else 1.0 / np.sqrt(D)
    return q, k, v, do, cu, T, Hq, Hkv, D, scale


def attn_rows(q, k, v, rows, do=None, cu_seqlens=None, softmax_scale=None):
    """Row pass on the given query rows.

    Returns dict with O [n,Hq,D], lse [Hq,n] and, when ``do`` is given,
    delta [Hq,n] and dQ [n,Hq,D].
    """
    lib = _load()
    q, k, v, do, cu, T, Hq, Hkv, D, scale = _prep(q, k, v, do, cu_seqlens, softmax_scale)
    rows = np.ascontiguousarray(rows, np.int64)
    n = rows.size
    assert n == 0 or (rows.min() >= 0 and rows.max() < T)
    O = np.zeros((n, Hq, D)); lse = np.zeros((Hq, n))
    delta = np.zeros((Hq, n)) if do is not None else None
    dQ = np.zeros((n, Hq, D)) if do is not None else None
    rc = lib.ref_attn_rows(_p(q), _p(k), _p(v), _p(do), _p(cu), ctypes.c_int32(cu.size - 1),
                           ctypes.c_int64(T), ctypes.c_int32(Hq), ctypes.c_int32(Hkv), ctypes.c_int32(D),
                           ctypes.c_double(scale), _p(rows), ctypes.c_int64(n),
                           _p(O), _p(lse), _p(delta), _p(dQ))
    if rc != 0:
        raise MemoryError("ref_attn_rows")
    out = dict(O=O, lse=lse)
    if do is not None:
        out.update(delta=delta, dQ=dQ)
    return out


def attn_cols(q, k, v, do, rows, lse_rows, delta_rows, cols, cu_seqlens=None, softmax_scale=None):
    """Column pass: dK, dV [n_cols,Hkv,D] summed over the participating ``rows`` (ascending)."""
    lib = _load()
    q, k, v, do, cu, T, Hq, Hkv, D, scale = _prep(q, k, v, do, cu_seqlens, softmax_scale)
    rows = np.ascontiguousarray(rows, np.int64); cols = np.ascontiguousarray(cols, np.int64)
    assert np.all(np.diff(rows) > 0)
    lse_rows = np.ascontiguousarray(lse_rows, np.float64); delta_rows = np.ascontiguousarray(delta_rows, np.float64)
    assert lse_rows.shape == delta_rows.shape == (Hq, rows.size)
    dK = np.zeros((cols.size, Hkv, D)); dV = np.zeros((cols.size, Hkv, D))
    lib.ref_attn_cols(_p(q), _p(k), _p(v), _p(do), _p(cu), ctypes.c_int32(cu.size - 1), ctypes.c_int64(T),
                      ctypes.c_int32(Hq), ctypes.c_int32(Hkv), ctypes.c_int32(D), ctypes.c_double(scale),
                      _p(rows), ctypes.c_int64(rows.size), _p(lse_rows), _p(delta_rows),
                      _p(cols), ctypes.c_int64(cols.size), _p(dK), _p(dV))
    return dK, dV


def attn_fwd(q, k, v, cu_seqlens=None, softmax_scale=None):
    """All rows: O [T,Hq,D], LSE [Hq,T]."""
    r = attn_rows(q, k, v, np.arange(q.shape[0]), None, cu_seqlens, softmax_scale)
    return r["O"], r["lse"]


def attn_bwd(q, k, v, do, cu_seqlens=None, softmax_scale=None):
    """All rows and columns: dQ, dK, dV, Delta."""
    T = q.shape[0]
    allr = np.arange(T)
    r = attn_rows(q, k, v, allr, do, cu_seqlens, softmax_scale)
    dK, dV = attn_cols(q, k, v, do, allr, r["lse"], r["delta"], allr, cu_seqlens, softmax_scale)
    return r["dQ"], dK, dV, r["delta"]
