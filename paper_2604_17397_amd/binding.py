"""ctypes binding of libsdvg.so. Argument marshalling only: same names as the C entry points.

PyTorch tensors supply device memory (`data_ptr()`) and the HIP stream; nothing is computed
here and there is no fallback: a missing library raises.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# SDVG_LIBRARY names another build of the same library (e.g. one with host sanitizers); there is
# still no fallback: whatever path is named must exist.
LIB_PATH = os.environ.get("SDVG_LIBRARY") or os.path.join(HERE, "libsdvg.so")

SDVG_BF16, SDVG_F32 = 0, 1
SDVG_SPLIT_NEVER, SDVG_SPLIT_AUTO, SDVG_SPLIT_ALWAYS = 0, 1, 2
_SPLIT = {"never": 0, "auto": 1, "always": 2}


class SdvgError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s failed: %s" % (where, status_string(status)))


class sdvg_kv_cache(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("n_layers", ctypes.c_int32), ("n_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block_tokens", ctypes.c_int32),
                ("capacity_tokens", ctypes.c_int64), ("cache_len", ctypes.c_int64),
                ("layer_stride", ctypes.c_int64), ("token_stride", ctypes.c_int64),
                ("head_stride", ctypes.c_int64)]


class sdvg_attn_desc(ctypes.Structure):
    _fields_ = [("n_q", ctypes.c_int32), ("n_blk", ctypes.c_int32),
                ("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("q_token_stride", ctypes.c_int64), ("q_head_stride", ctypes.c_int64),
                ("o_token_stride", ctypes.c_int64), ("o_head_stride", ctypes.c_int64),
                ("kv_token_stride", ctypes.c_int64), ("kv_head_stride", ctypes.c_int64),
                ("blk_token_stride", ctypes.c_int64), ("blk_head_stride", ctypes.c_int64),
                ("scale", ctypes.c_float), ("dtype", ctypes.c_int32)]


_LIB = None


def lib():
    """The loaded libsdvg.so; raises if it was never built."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libsdvg.so is missing: build it with `python -m paper_2604_17397_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
        L.sdvg_block_attn.restype = ctypes.c_int
        L.sdvg_block_attn.argtypes = [ctypes.POINTER(sdvg_attn_desc), vp, vp, vp, vp, vp, i64, vp, vp]
        L.sdvg_block_attn_commit.restype = ctypes.c_int
        L.sdvg_block_attn_commit.argtypes = [ctypes.POINTER(sdvg_attn_desc), vp, vp, vp, vp, vp, i64, vp, vp]
        L.sdvg_kv_commit_mark.restype = ctypes.c_int
        L.sdvg_kv_commit_mark.argtypes = [ctypes.POINTER(sdvg_kv_cache), i32]
        pp = ctypes.POINTER(ctypes.c_void_p)
        L.sdvg_block_attn_batch.restype = ctypes.c_int
        L.sdvg_block_attn_batch.argtypes = [ctypes.POINTER(sdvg_attn_desc), i32, pp, pp, pp, pp, pp, i64, pp,
                                            vp, i64, i32, vp]
        L.sdvg_block_attn_batch_static.restype = ctypes.c_int
        L.sdvg_block_attn_batch_static.argtypes = [ctypes.POINTER(sdvg_attn_desc), i32, pp, pp, pp, pp, pp, i64, pp,
                                                   i32, vp]
        L.sdvg_block_attn_static_workspace_limit.restype = ctypes.c_int64
        L.sdvg_block_attn_workspace_bytes.restype = ctypes.c_int64
        L.sdvg_block_attn_workspace_bytes.argtypes = [ctypes.POINTER(sdvg_attn_desc), i32, i64, i32]
        L.sdvg_kv_commit.restype = ctypes.c_int
        L.sdvg_kv_commit.argtypes = [ctypes.POINTER(sdvg_kv_cache), vp, vp, i32, vp]
        L.sdvg_rope.restype = ctypes.c_int
        L.sdvg_rope.argtypes = [vp, vp, vp, vp, i64, i32, i32, i64, i64, i64, i64, vp]
        L.sdvg_kv_commit_rope.restype = ctypes.c_int
        L.sdvg_kv_commit_rope.argtypes = [ctypes.POINTER(sdvg_kv_cache), vp, vp, i32, vp, vp, vp]
        L.sdvg_kv_rollback.restype = ctypes.c_int
        L.sdvg_kv_rollback.argtypes = [ctypes.POINTER(sdvg_kv_cache), i64, vp]
        L.sdvg_worst_frame_route.restype = ctypes.c_int
        L.sdvg_worst_frame_route.argtypes = [vp, i32, f32, i32, ctypes.POINTER(f32), vp]
        L.sdvg_worst_frame_route_batch.restype = ctypes.c_int
        L.sdvg_worst_frame_route_batch.argtypes = [vp, i32, i32, f32, vp, i32, vp, vp, vp]
        L.sdvg_buffer_snapshot.restype = ctypes.c_int
        L.sdvg_buffer_snapshot.argtypes = [vp, vp, i64, vp]
        L.sdvg_avg_frame_route.restype = ctypes.c_int
        L.sdvg_avg_frame_route.argtypes = [vp, i32, f32, i32, ctypes.POINTER(f32), vp]
        L.sdvg_avg_frame_route_batch.restype = ctypes.c_int
        L.sdvg_avg_frame_route_batch.argtypes = [vp, i32, i32, f32, vp, i32, vp, vp, vp]
        L.sdvg_probe_mfma.restype = ctypes.c_int
        L.sdvg_probe_mfma.argtypes = [vp, i64, vp, i32, ctypes.POINTER(ctypes.c_double), vp]
        L.sdvg_probe_mfma_changing.restype = ctypes.c_int
        L.sdvg_probe_mfma_changing.argtypes = [vp, i64, vp, i32, ctypes.POINTER(ctypes.c_double), vp]
        L.sdvg_status_string.restype = ctypes.c_char_p
        L.sdvg_status_string.argtypes = [ctypes.c_int]
        L.sdvg_last_device_error.restype = ctypes.c_int
        L.sdvg_version.restype = ctypes.c_int
        L.sdvg_shutdown.restype = None
        _LIB = L
    return _LIB


def status_string(status):
    return lib().sdvg_status_string(int(status)).decode()


def _stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _check_dev(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("libsdvg takes device tensors")


class KVCache:
    """Caller-owned KV cache of one model: k, v are bf16 device tensors whose logical view is
    [layers, capacity_tokens, heads, 128] (any layer/token/head strides, unit dim stride)."""

    def __init__(self, k, v, block_tokens, cache_len=0):
        _check_dev(k, v)
        assert k.dtype == torch.bfloat16 and v.dtype == torch.bfloat16
        assert k.dim() == 4 and k.shape == v.shape and k.stride() == v.stride() and k.stride(3) == 1
        self.k, self.v = k, v
        self.c = sdvg_kv_cache(k.data_ptr(), v.data_ptr(), k.shape[0], k.shape[2], k.shape[3],
                               int(block_tokens), k.shape[1], int(cache_len),
                               k.stride(0), k.stride(1), k.stride(2))

    @property
    def cache_len(self):
        return int(self.c.cache_len)

    def layer(self, i):
        """(k, v) views [capacity, heads, 128] of layer i."""
        return self.k[i], self.v[i]


def _attn_desc(q, k_cache, v_cache, k_blk, v_blk, cache_len, out, scale):
    """Checks one (q, cache, block, out) set and returns its descriptor. Shapes are checked
    against each other here, because a wrong length or head count would make the kernel read
    outside the tensors."""
    _check_dev(q, k_cache, v_cache, k_blk, v_blk, out)
    if q.dtype == torch.bfloat16:
        dtype = SDVG_BF16
    elif q.dtype == torch.float32:
        dtype = SDVG_F32
    else:
        raise TypeError("q must be bfloat16 or float32")
    if q.dim() != 3 or q.stride(2) != 1:
        raise ValueError("q must be 3-d with unit dim stride")
    if (k_cache is None) != (v_cache is None):
        raise ValueError("k_cache and v_cache come together")
    for t in (k_cache, v_cache, k_blk, v_blk):
        if t is not None and (t.dtype != q.dtype or t.dim() != 3 or t.stride(2) != 1):
            raise ValueError("all tensors share q's dtype, are 3-d and have unit dim stride")
        if t is not None and (t.shape[1] != q.shape[1] or t.shape[2] != q.shape[2]):
            raise ValueError("all tensors share q's head count and head_dim")
        if t is not None and t.device != q.device:
            raise ValueError("all tensors live on q's device")
    if v_blk.shape != k_blk.shape:
        raise ValueError("k_blk and v_blk must have the same shape")
    if cache_len < 0 or (cache_len > 0 and k_cache is None):
        raise ValueError("cache_len is negative, or positive without a cache")
    if k_cache is not None and (v_cache.shape != k_cache.shape or cache_len > k_cache.shape[0]):
        raise ValueError("cache_len exceeds the cache tensors (or k_cache / v_cache differ in shape)")
    if (out.shape != q.shape or out.dtype != q.dtype or out.stride(2) != 1 or out.device != q.device):
        raise ValueError("out must match q in shape, dtype and device and have unit dim stride")
    if k_blk.stride() != v_blk.stride() or (k_cache is not None and k_cache.stride() != v_cache.stride()):
        raise ValueError("k and v must share strides")
    kv_ts, kv_hs = (k_cache.stride(0), k_cache.stride(1)) if k_cache is not None else (128, 128)
    return sdvg_attn_desc(q.shape[0], k_blk.shape[0], q.shape[1], q.shape[2],
                          q.stride(0), q.stride(1), out.stride(0), out.stride(1),
                          kv_ts, kv_hs, k_blk.stride(0), k_blk.stride(1),
                          0.0 if scale is None else float(scale), dtype)


def block_attn(q, k_cache, v_cache, k_blk, v_blk, cache_len, out=None, scale=None, stream=None):
    """sdvg_block_attn: q, k_blk, v_blk [tokens, heads, 128]; k_cache, v_cache one layer's
    [>= cache_len, heads, 128] (may be None when cache_len == 0). `scale=None` passes 0, which the
    library reads as 1/sqrt(head_dim). Returns out."""
    cache_len = int(cache_len)
    if out is None:
        out = torch.empty(q.shape, dtype=q.dtype, device=q.device)
    d = _attn_desc(q, k_cache, v_cache, k_blk, v_blk, cache_len, out, scale)
    st = lib().sdvg_block_attn(ctypes.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_blk),
                               _ptr(v_blk), cache_len, _ptr(out), _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_block_attn")
    return out


def block_attn_commit(q, k_cache, v_cache, k_blk, v_blk, cache_len, out=None, scale=None, stream=None):
    """sdvg_block_attn_commit: block_attn for one layer that also copies k_blk / v_blk into tokens
    [cache_len, cache_len + n_blk) of k_cache / v_cache (which must be long enough). Returns out."""
    cache_len = int(cache_len)
    if out is None:
        out = torch.empty(q.shape, dtype=q.dtype, device=q.device)
    if k_cache is None or v_cache is None:
        raise ValueError("the fused commit needs the layer's cache tensors")
    d = _attn_desc(q, k_cache, v_cache, k_blk, v_blk, cache_len, out, scale)
    if cache_len + k_blk.shape[0] > k_cache.shape[0]:
        raise ValueError("the cache has no room for the block after cache_len")
    st = lib().sdvg_block_attn_commit(ctypes.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(k_blk),
                                      _ptr(v_blk), cache_len, _ptr(out), _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_block_attn_commit")
    return out


def kv_commit_mark(cache, slot):
    st = lib().sdvg_kv_commit_mark(ctypes.byref(cache.c), int(slot))
    if st != 0:
        raise SdvgError(st, "sdvg_kv_commit_mark")


def _desc_key(d):
    return tuple(getattr(d, f) for f, _ in d._fields_)


def block_attn_workspace_bytes(q, k_cache, v_cache, k_blk, v_blk, cache_len, n_items=1, split="auto", scale=None):
    """sdvg_block_attn_workspace_bytes for the shape of these tensors; split is "never", "auto" or
    "always"."""
    cache_len = int(cache_len)
    d = _attn_desc(q, k_cache, v_cache, k_blk, v_blk, cache_len, q, scale)
    n = lib().sdvg_block_attn_workspace_bytes(ctypes.byref(d), int(n_items), cache_len, _SPLIT[split])
    if n < 0:
        raise SdvgError(n, "sdvg_block_attn_workspace_bytes")
    return int(n)


def block_attn_batch_static(qs, k_caches, v_caches, k_blks, v_blks, cache_len, outs, split="auto", scale=None,
                            stream=None):
    """sdvg_block_attn_batch_static: as block_attn_batch, with the library's fixed workspace. `outs`
    is required (this entry point is for callers that do not allocate)."""
    return block_attn_batch(qs, k_caches, v_caches, k_blks, v_blks, cache_len, outs=outs, split=split, scale=scale,
                            stream=stream, _static=True)


def block_attn_batch(qs, k_caches, v_caches, k_blks, v_blks, cache_len, outs=None, workspace=None,
                     split="auto", scale=None, stream=None, _static=False):
    """sdvg_block_attn_batch: lists of n tensors each (k_caches / v_caches may be None when
    cache_len == 0); every item must have the same shapes and strides. `workspace`: optional
    device tensor (any dtype) the library may use to split keys over workgroups, under the policy
    `split` ("never", "auto", "always"). Returns outs."""
    cache_len = int(cache_len)
    n = len(qs)
    if k_caches is None:
        k_caches, v_caches = [None] * n, [None] * n
    if not (len(k_caches) == len(v_caches) == len(k_blks) == len(v_blks) == n):
        raise ValueError("every list needs one tensor per item")
    if outs is None:
        outs = [torch.empty(q.shape, dtype=q.dtype, device=q.device) for q in qs]
    descs = [_attn_desc(qs[i], k_caches[i], v_caches[i], k_blks[i], v_blks[i], cache_len, outs[i], scale)
             for i in range(n)]
    if any(_desc_key(d) != _desc_key(descs[0]) for d in descs[1:]):
        raise ValueError("all items of a batch must share shapes, strides and dtype")
    if any(t.device != qs[0].device for t in qs):
        raise ValueError("all items live on one device")

    def arr(ts):
        return (ctypes.c_void_p * n)(*[t.data_ptr() if t is not None else None for t in ts])
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        _check_dev(workspace)
        if not workspace.is_contiguous() or workspace.device != qs[0].device:
            raise ValueError("workspace must be a contiguous tensor on the items' device")
        ws_ptr, ws_bytes = _ptr(workspace), workspace.numel() * workspace.element_size()
    if _static:
        st = lib().sdvg_block_attn_batch_static(ctypes.byref(descs[0]), n, arr(qs), arr(k_caches), arr(v_caches),
                                                arr(k_blks), arr(v_blks), cache_len, arr(outs), _SPLIT[split],
                                                _stream_ptr(stream))
    else:
        st = lib().sdvg_block_attn_batch(ctypes.byref(descs[0]), n, arr(qs), arr(k_caches), arr(v_caches),
                                         arr(k_blks), arr(v_blks), cache_len, arr(outs), ws_ptr, ws_bytes,
                                         _SPLIT[split], _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_block_attn_batch_static" if _static else "sdvg_block_attn_batch")
    return outs


def kv_commit(cache, k_blk, v_blk, slot, stream=None):
    """sdvg_kv_commit: k_blk, v_blk dense bf16 [layers, T, heads, 128]."""
    _check_dev(k_blk, v_blk)
    if not (k_blk.is_contiguous() and v_blk.is_contiguous()):
        raise ValueError("k_blk and v_blk must be dense")
    L, T, H, D = cache.c.n_layers, cache.c.block_tokens, cache.c.n_heads, cache.c.head_dim
    if tuple(k_blk.shape) != (L, T, H, D) or tuple(v_blk.shape) != (L, T, H, D):
        raise ValueError("block shape must be [layers, T, heads, dim] of the cache")
    if k_blk.dtype != torch.bfloat16 or v_blk.dtype != torch.bfloat16:
        raise TypeError("k_blk and v_blk must be bfloat16")
    st = lib().sdvg_kv_commit(ctypes.byref(cache.c), _ptr(k_blk), _ptr(v_blk), int(slot),
                              _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_kv_commit")


def _check_tables(cos, sin, n_tokens, device):
    _check_dev(cos, sin)
    for t in (cos, sin):
        if t.dtype != torch.float32 or tuple(t.shape) != (n_tokens, 64) or not t.is_contiguous() or t.device != device:
            raise ValueError("cos / sin must be dense float32 [tokens, 64] on the tensors' device")


def rope(x, cos, sin, out=None, stream=None):
    """sdvg_rope: rotary embedding of bf16 rows x [tokens, heads, 128] by the angle tables cos, sin
    float32 [tokens, 64]. out defaults to a new tensor; pass out=x for in place."""
    _check_dev(x, out)
    if x.dtype != torch.bfloat16 or x.dim() != 3 or x.shape[2] != 128 or x.stride(2) != 1:
        raise ValueError("x must be bfloat16 [tokens, heads, 128] with unit dim stride")
    if out is None:
        out = torch.empty(x.shape, dtype=x.dtype, device=x.device)
    elif out.shape != x.shape or out.dtype != x.dtype or out.stride(2) != 1 or out.device != x.device:
        raise ValueError("out must match x")
    _check_tables(cos, sin, x.shape[0], x.device)
    st = lib().sdvg_rope(_ptr(x), _ptr(cos), _ptr(sin), _ptr(out), x.shape[0], x.shape[1], x.shape[2],
                         x.stride(0), x.stride(1), out.stride(0), out.stride(1), _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_rope")
    return out


def kv_commit_rope(cache, k_blk, v_blk, slot, cos, sin, stream=None):
    """sdvg_kv_commit_rope: kv_commit with k_blk (dense bf16 [layers, T, heads, 128], BEFORE the
    rotary embedding) rotated on its way into the cache; cos, sin float32 [T, 64]."""
    _check_dev(k_blk, v_blk)
    if not (k_blk.is_contiguous() and v_blk.is_contiguous()):
        raise ValueError("k_blk and v_blk must be dense")
    L, T, H, D = cache.c.n_layers, cache.c.block_tokens, cache.c.n_heads, cache.c.head_dim
    if tuple(k_blk.shape) != (L, T, H, D) or tuple(v_blk.shape) != (L, T, H, D):
        raise ValueError("block shape must be [layers, T, heads, dim] of the cache")
    if k_blk.dtype != torch.bfloat16 or v_blk.dtype != torch.bfloat16:
        raise TypeError("k_blk and v_blk must be bfloat16")
    _check_tables(cos, sin, T, k_blk.device)
    st = lib().sdvg_kv_commit_rope(ctypes.byref(cache.c), _ptr(k_blk), _ptr(v_blk), int(slot), _ptr(cos), _ptr(sin),
                                   _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_kv_commit_rope")


def kv_rollback(cache, new_len, stream=None):
    st = lib().sdvg_kv_rollback(ctypes.byref(cache.c), int(new_len), _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_kv_rollback")


def buffer_snapshot(dst, src, n_bytes=None, stream=None):
    """sdvg_buffer_snapshot: dst[:n_bytes] = src[:n_bytes] for two device tensors viewed as bytes
    (n_bytes defaults to the size of src)."""
    _check_dev(dst, src)
    if not (dst.is_contiguous() and src.is_contiguous()):
        raise ValueError("buffer_snapshot needs contiguous tensors")
    if n_bytes is None:
        n_bytes = src.numel() * src.element_size()
    if n_bytes > dst.numel() * dst.element_size() or n_bytes > src.numel() * src.element_size():
        raise ValueError("n_bytes exceeds a buffer")
    st = lib().sdvg_buffer_snapshot(_ptr(dst), _ptr(src), int(n_bytes), _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_buffer_snapshot")


def worst_frame_route(frame_scores, tau, block_idx, stream=None, mode="min"):
    """sdvg_worst_frame_route (mode "min") or sdvg_avg_frame_route (mode "mean"): returns
    (decision, q_b) with q_b a numpy float32 scalar."""
    import numpy as np
    fn = {"min": lib().sdvg_worst_frame_route, "mean": lib().sdvg_avg_frame_route}[mode]
    _check_dev(frame_scores)
    if frame_scores.dtype != torch.float32 or frame_scores.dim() != 1 or not frame_scores.is_contiguous():
        raise ValueError("frame_scores must be a dense 1-d float32 tensor")
    qb = np.zeros(1, dtype=np.float32)
    st = fn(_ptr(frame_scores), frame_scores.numel(), float(tau), int(block_idx),
            qb.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), _stream_ptr(stream))
    if st < 0:
        raise SdvgError(st, "sdvg_worst_frame_route")
    return int(st), qb[0]


def worst_frame_route_batch(frame_scores, tau, block_idx=None, first_block_idx=0, stream=None, mode="min"):
    """sdvg_worst_frame_route_batch (mode "min") or sdvg_avg_frame_route_batch (mode "mean"):
    frame_scores [n_blocks, n_frames] fp32; returns device tensors (decisions int32 [n_blocks],
    q_b float32 [n_blocks]). Asynchronous."""
    fn = {"min": lib().sdvg_worst_frame_route_batch, "mean": lib().sdvg_avg_frame_route_batch}[mode]
    _check_dev(frame_scores, block_idx)
    if frame_scores.dtype != torch.float32 or frame_scores.dim() != 2 or not frame_scores.is_contiguous():
        raise ValueError("frame_scores must be a dense 2-d float32 tensor")
    n_blocks, n_frames = frame_scores.shape
    if block_idx is not None and (block_idx.dtype != torch.int32 or block_idx.numel() != n_blocks):
        raise ValueError("block_idx must be int32 [n_blocks]")
    dec = torch.empty(n_blocks, dtype=torch.int32, device=frame_scores.device)
    qb = torch.empty(n_blocks, dtype=torch.float32, device=frame_scores.device)
    st = fn(_ptr(frame_scores), n_blocks, n_frames, float(tau), _ptr(block_idx), int(first_block_idx),
            _ptr(dec), _ptr(qb), _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, "sdvg_worst_frame_route_batch")
    return dec, qb


def probe_mfma(iters=20000, stream=None, changing=False):
    """sdvg_probe_mfma (or, with changing=True, sdvg_probe_mfma_changing): enqueues the MFMA-only
    measurement kernel. Returns (flops, cycles) with cycles a device uint64 tensor (as int64)
    holding wave 0's shader clocks once it has run."""
    dev = torch.device("cuda", torch.cuda.current_device())
    out = torch.empty(256 * 256, dtype=torch.float32, device=dev)
    cycles = torch.zeros(1, dtype=torch.int64, device=dev)
    flops = ctypes.c_double(0.0)
    name = "sdvg_probe_mfma_changing" if changing else "sdvg_probe_mfma"
    st = getattr(lib(), name)(_ptr(out), out.numel(), _ptr(cycles), int(iters), ctypes.byref(flops),
                              _stream_ptr(stream))
    if st != 0:
        raise SdvgError(st, name)
    return flops.value, cycles
