"""ctypes front-end of the plain-C oracle (oracle/sdvg_oracle.c).

Test infrastructure, not the product. Inputs are numpy arrays holding exactly the bits the
GPU path sees: bf16 tensors as uint16 bit patterns, fp32 tensors as float32. Outputs are fp64.
Logical index order everywhere: (layer, token, head, dim).
"""
import ctypes
import math
import os

import numpy as np

from . import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.build(force=False)
        lib = ctypes.CDLL(path)
        i64, dbl, vp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.sdvg_oracle_block_attn.restype = ctypes.c_int
        lib.sdvg_oracle_block_attn.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int,
                                               i64, i64, i64, i64,
                                               i64, i64, i64, i64, i64, i64,
                                               dbl, vp, i64, vp, vp]
        lib.sdvg_oracle_kv_commit.restype = ctypes.c_int
        lib.sdvg_oracle_kv_commit.argtypes = [vp, vp, i64, i64, i64, i64, i64,
                                              ctypes.POINTER(i64), vp, vp, i64]
        lib.sdvg_oracle_kv_rollback.restype = ctypes.c_int
        lib.sdvg_oracle_kv_rollback.argtypes = [vp, vp, i64, i64, i64, i64,
                                                ctypes.POINTER(i64), i64]
        lib.sdvg_oracle_buffer_copy.restype = ctypes.c_int
        lib.sdvg_oracle_buffer_copy.argtypes = [vp, vp, i64]
        lib.sdvg_oracle_route.restype = ctypes.c_int
        lib.sdvg_oracle_route.argtypes = [vp, i64, ctypes.c_float, i64, ctypes.c_int, vp]
        lib.sdvg_oracle_rope.restype = ctypes.c_int
        lib.sdvg_oracle_rope.argtypes = [vp, vp, vp, vp, i64, i64, i64]
        lib.sdvg_oracle_num_threads.restype = ctypes.c_int
        _LIB = lib
    return _LIB


def num_threads() -> int:
    return int(_lib().sdvg_oracle_num_threads())


def _elem_stride(a, axis):
    assert a.strides[axis] % a.itemsize == 0
    return a.strides[axis] // a.itemsize


def _dtype_code(a):
    if a.dtype == np.uint16:
        return 0
    if a.dtype == np.float32:
        return 1
    raise TypeError("oracle takes bf16 bit patterns (uint16) or float32, got %s" % a.dtype)


def block_attn(q, k_cache, v_cache, k_blk, v_blk, cache_len, scale=None, rows=None,
               return_weights=False):
    """softmax(q [cache[:cache_len]; blk]^T * scale) [cache; blk] per head, fp64.

    q, k_blk, v_blk: [tokens, heads, dim]; k_cache, v_cache: [>= cache_len, heads, dim]
    (any token/head strides, unit dim stride). rows: optional list of query rows to compute.
    Returns out [n_rows, heads, dim] (and the normalised weights [n_rows, heads, n_k]).
    """
    code = _dtype_code(q)
    for a in (k_cache, v_cache, k_blk, v_blk):
        assert _dtype_code(a) == code
        assert a.ndim == 3 and a.strides[2] == a.itemsize
    assert q.ndim == 3 and q.strides[2] == q.itemsize
    n_q, n_heads, head_dim = q.shape
    n_blk = k_blk.shape[0]
    assert k_blk.shape == v_blk.shape and k_blk.shape[1:] == (n_heads, head_dim)
    assert k_cache.shape[0] >= cache_len and v_cache.shape[0] >= cache_len
    assert k_cache.strides == v_cache.strides and k_blk.strides == v_blk.strides
    if scale is None:
        scale = 1.0 / math.sqrt(float(head_dim))
    if rows is None:
        rows_arr, rows_ptr, n_rows = None, None, n_q
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        assert rows_arr.size == 0 or (rows_arr.min() >= 0 and rows_arr.max() < n_q)
        rows_ptr, n_rows = rows_arr.ctypes.data, rows_arr.size
    out = np.empty((n_rows, n_heads, head_dim), dtype=np.float64)
    n_k = cache_len + n_blk
    weights = np.empty((n_rows, n_heads, n_k), dtype=np.float64) if return_weights else None
    rc = _lib().sdvg_oracle_block_attn(
        q.ctypes.data, k_cache.ctypes.data, v_cache.ctypes.data, k_blk.ctypes.data,
        v_blk.ctypes.data, code, n_blk, n_heads, head_dim, cache_len,
        _elem_stride(q, 0), _elem_stride(q, 1),
        _elem_stride(k_cache, 0), _elem_stride(k_cache, 1),
        _elem_stride(k_blk, 0), _elem_stride(k_blk, 1),
        float(scale), rows_ptr, n_rows, out.ctypes.data,
        weights.ctypes.data if return_weights else None)
    if rc != 0:
        raise RuntimeError("sdvg_oracle_block_attn failed: %d" % rc)
    return (out, weights) if return_weights else out


class KVMirror:
    """Host mirror of the KV cache: k, v are uint16 [layers, capacity, heads, dim], dense."""

    def __init__(self, n_layers, capacity_tokens, n_heads, head_dim, block_tokens, fill=0):
        shape = (n_layers, capacity_tokens, n_heads, head_dim)
        self.k = np.full(shape, fill, dtype=np.uint16)
        self.v = np.full(shape, fill, dtype=np.uint16)
        self.block_tokens = int(block_tokens)
        self.cache_len = 0


def kv_commit(mirror, k_blk, v_blk, slot):
    """Append block [layers, T, heads, dim] (uint16) into slot; returns the C status."""
    L, cap, H, d = mirror.k.shape
    T = mirror.block_tokens
    assert k_blk.dtype == np.uint16 and v_blk.dtype == np.uint16
    assert k_blk.shape == (L, T, H, d) and v_blk.shape == (L, T, H, d)
    k_blk = np.ascontiguousarray(k_blk)
    v_blk = np.ascontiguousarray(v_blk)
    n = ctypes.c_int64(mirror.cache_len)
    rc = _lib().sdvg_oracle_kv_commit(mirror.k.ctypes.data, mirror.v.ctypes.data, L, cap, H, d,
                                      T, ctypes.byref(n), k_blk.ctypes.data, v_blk.ctypes.data,
                                      int(slot))
    mirror.cache_len = int(n.value)
    return rc


def kv_rollback(mirror, new_len):
    L, cap, H, d = mirror.k.shape
    n = ctypes.c_int64(mirror.cache_len)
    rc = _lib().sdvg_oracle_kv_rollback(mirror.k.ctypes.data, mirror.v.ctypes.data, L, cap, H, d,
                                        ctypes.byref(n), int(new_len))
    mirror.cache_len = int(n.value)
    return rc


def buffer_copy(dst, src, n_bytes=None):
    """dst[:n_bytes] = src[:n_bytes] on two contiguous uint8 arrays, in place; returns the C status."""
    assert dst.dtype == np.uint8 and src.dtype == np.uint8
    assert dst.flags.c_contiguous and src.flags.c_contiguous
    if n_bytes is None:
        n_bytes = src.size
    assert n_bytes <= dst.size and n_bytes <= src.size
    return _lib().sdvg_oracle_buffer_copy(dst.ctypes.data, src.ctypes.data, int(n_bytes))


def route(scores, tau, block_idx, mode="min"):
    """Returns (decision, q_b) with q_b a numpy float32 scalar."""
    s = np.ascontiguousarray(scores, dtype=np.float32)
    assert s.ndim == 1 and s.size >= 1
    qb = np.zeros(1, dtype=np.float32)  # array, so a NaN payload survives bit for bit
    dec = _lib().sdvg_oracle_route(s.ctypes.data, s.size, ctypes.c_float(tau), int(block_idx),
                                   {"min": 0, "mean": 1}[mode], qb.ctypes.data)
    return int(dec), qb[0]


def rope(x, cos, sin):
    """Rotary embedding of bf16 rows x [tokens, heads, dim] (uint16 bit patterns) by the angles
    whose cosines / sines are given per (token, pair): cos, sin float32 [tokens, dim // 2].
    Returns uint16 bit patterns of the same shape."""
    assert x.dtype == np.uint16 and x.ndim == 3
    x = np.ascontiguousarray(x)
    n, H, d = x.shape
    cos = np.ascontiguousarray(cos, dtype=np.float32)
    sin = np.ascontiguousarray(sin, dtype=np.float32)
    assert cos.shape == (n, d // 2) and sin.shape == (n, d // 2)
    out = np.empty_like(x)
    rc = _lib().sdvg_oracle_rope(x.ctypes.data, cos.ctypes.data, sin.ctypes.data, out.ctypes.data, n, H, d)
    if rc != 0:
        raise RuntimeError("sdvg_oracle_rope failed: %d" % rc)
    return out
