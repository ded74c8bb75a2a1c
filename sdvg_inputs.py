"""Seeded synthetic inputs for the SDVG attention / KV-cache / routing path.

This module serves both the CPU oracle's tests and the GPU path's tests and benchmark. It
holds none of the method's arithmetic: only a counter-based random generator, the
float -> bfloat16 bit conversion of the *inputs*, and the workload shapes.

Generator: value i of tensor `tensor_id` under `seed` comes from a splitmix64 hash of a
counter, so any element can be regenerated independently of the others. Normal variates are
Box-Muller in fp64 from two hashed uniforms.

Workload shapes stand in for the paper's 832x480 protocol (Sec. 4.1 "Generation protocol":
3 latent frames per block, 12 decoded frames scored per later block, seed 42): 30x52 latent
tokens per frame -> 4680 tokens per block, head_dim 128, 12 heads (1.3B drafter) or 40 heads
(14B target).
"""
import math

import numpy as np

SEED = 42  # the paper's fixed seed (Sec. 4.1 "Generation protocol")

# tensor ids (per-layer tensors add 100 * layer)
TID_Q, TID_K_CACHE, TID_V_CACHE, TID_K_BLK, TID_V_BLK, TID_SCORES, TID_HEAD_SCALE = range(7)

CONFIGS = {
    # name: heads, block tokens, cached blocks, layers
    "tiny": dict(n_heads=12, head_dim=128, block_tokens=3 * 8 * 13, cached_blocks=2, n_layers=1),
    "drafter": dict(n_heads=12, head_dim=128, block_tokens=3 * 30 * 52, cached_blocks=2,
                    n_layers=30),
    "target": dict(n_heads=40, head_dim=128, block_tokens=3 * 30 * 52, cached_blocks=6,
                   n_layers=40),
}

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z):
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _stream_key(seed, tensor_id):
    with np.errstate(over="ignore"):
        k = _mix(np.uint64(seed) * _GOLDEN + np.uint64(tensor_id) + np.uint64(1))
        return _mix(k * _GOLDEN + np.uint64(tensor_id))


def uniform_bits(seed, tensor_id, start, count):
    """uint64 hash of counters start .. start+count-1 in stream (seed, tensor_id)."""
    with np.errstate(over="ignore"):
        ctr = np.arange(start, start + count, dtype=np.uint64)
        return _mix(_stream_key(seed, tensor_id) + (ctr + np.uint64(1)) * _GOLDEN)


def normal(seed, tensor_id, count, start=0, chunk=1 << 22):
    """count standard normal fp64 variates, element i from counters 2i and 2i+1."""
    out = np.empty(count, dtype=np.float64)
    for lo in range(0, count, chunk):
        n = min(chunk, count - lo)
        bits = uniform_bits(seed, tensor_id, 2 * (start + lo), 2 * n)
        u1 = ((bits[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
        u2 = (bits[1::2] >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
        out[lo:lo + n] = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    return out


def uniform(seed, tensor_id, count, lo=0.0, hi=1.0, start=0):
    bits = uniform_bits(seed, tensor_id, start, count)
    u = (bits >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
    return lo + (hi - lo) * u


def f32_to_bf16_bits(x):
    """float32 array -> bfloat16 bit patterns (uint16), round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f64(bits):
    """bfloat16 bit patterns -> float64 (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def normal_bf16(seed, tensor_id, shape, head_scale=None):
    """N(0,1) tensor [tokens, heads, dim] as bf16 bits; optional per-head fp32 multiplier."""
    x = normal(seed, tensor_id, int(np.prod(shape))).astype(np.float32).reshape(shape)
    if head_scale is not None:
        x = x * np.asarray(head_scale, dtype=np.float32).reshape(1, -1, 1)
    return f32_to_bf16_bits(x)


def normal_f32(seed, tensor_id, shape):
    return normal(seed, tensor_id, int(np.prod(shape))).astype(np.float32).reshape(shape)


def head_scales(seed, n_heads, which):
    """Per-head jitter U(0.5, 2), one independent draw per head per tensor (which = 0 q, 1 k, 2 v)."""
    return uniform(seed, TID_HEAD_SCALE, n_heads, 0.5, 2.0, start=which * n_heads).astype(np.float32)


def attn_inputs(n_heads, block_tokens, cache_len, head_dim=128, seed=SEED, jitter=False,
                dtype="bf16", cache_capacity=None, layer=0):
    """q, k_cache, v_cache, k_blk, v_blk for one layer.

    Cache arrays have cache_capacity tokens (default cache_len); tokens past cache_len are
    filled with NaN bit patterns so that any read past cache_len poisons the output.
    """
    cap = cache_len if cache_capacity is None else cache_capacity
    assert cap >= cache_len
    off = 100 * layer
    sq = sk = sv = None
    if jitter:
        sq, sk, sv = (head_scales(seed, n_heads, w) for w in range(3))
    if dtype == "bf16":
        gen = lambda tid, n, s: normal_bf16(seed, tid + off, (n, n_heads, head_dim), s)
        poison = np.uint16(0x7FC1)
        store = np.uint16
    else:
        def gen(tid, n, s):
            x = normal_f32(seed, tid + off, (n, n_heads, head_dim))
            return x if s is None else x * np.asarray(s, np.float32).reshape(1, -1, 1)
        poison = np.float32(np.nan)
        store = np.float32
    q = gen(TID_Q, block_tokens, sq)
    k_blk = gen(TID_K_BLK, block_tokens, sk)
    v_blk = gen(TID_V_BLK, block_tokens, sv)
    k_cache = np.full((cap, n_heads, head_dim), poison, dtype=store)
    v_cache = np.full((cap, n_heads, head_dim), poison, dtype=store)
    if cache_len:
        k_cache[:cache_len] = gen(TID_K_CACHE, cache_len, sk)
        v_cache[:cache_len] = gen(TID_V_CACHE, cache_len, sv)
    return q, k_cache, v_cache, k_blk, v_blk


def frame_scores_iid(seed, n_blocks, n_frames=12, mean=-0.3, std=0.6, tensor_id=TID_SCORES):
    """ImageReward-like per-frame scores, i.i.d. N(mean, std) per frame, fp32 [n_blocks, n_frames]."""
    z = normal(seed, tensor_id, n_blocks * n_frames)
    return (mean + std * z).astype(np.float32).reshape(n_blocks, n_frames)


def frame_scores_correlated(seed, n_blocks, n_frames=12, mean=-0.3, std=0.6, jitter=0.1,
                            tensor_id=TID_SCORES):
    """Block mean ~N(mean, std) plus per-frame jitter N(0, jitter): frames of a block move together."""
    mu = mean + std * normal(seed, tensor_id + 50, n_blocks)
    z = normal(seed, tensor_id + 51, n_blocks * n_frames).reshape(n_blocks, n_frames)
    return (mu[:, None] + jitter * z).astype(np.float32)


def parity_rows(n_q, head=64, tail=136, every=37):
    """Row sample for large shapes: first `head`, last `tail`, and every `every`-th row."""
    rows = set(range(min(head, n_q))) | set(range(max(0, n_q - tail), n_q)) | set(range(0, n_q, every))
    return np.array(sorted(rows), dtype=np.int64)


def attn_flops(n_q, n_k, n_heads, head_dim=128):
    """Algorithmic FLOPs of one attention call: QK^T and PV, 2 per multiply-add."""
    return 4.0 * n_q * n_k * head_dim * n_heads


# ---------------------------------------------------------------- device-side generation
# The numpy generator above is too slow for the full-size shapes (10^8..10^9 elements); the
# full-size GPU tests and the benchmark draw N(0,1) with torch's seeded generator on the device
# and copy the bits back for the oracle, so both sides still see identical inputs.

def device_normal_bf16(shape, seed, tensor_id, device="cuda", head_scale=None, chunk=1 << 26):
    """N(0,1) bfloat16 tensor of `shape` on `device`; optional per-head fp32 multiplier
    (shape[-2] must be the head axis). Filled in chunks to bound the fp32 temporary."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed) * 1000003 + int(tensor_id))
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    flat = out.view(-1)
    scale = None
    if head_scale is not None:
        scale = torch.as_tensor(np.asarray(head_scale, np.float32), device=device)
    inner = shape[-1] * shape[-2] if len(shape) >= 2 else 1
    step = max(inner, (chunk // inner) * inner)
    for lo in range(0, flat.numel(), step):
        n = min(step, flat.numel() - lo)
        x = torch.randn(n, generator=gen, device=device, dtype=torch.float32)
        if scale is not None:
            x = (x.view(-1, shape[-2], shape[-1]) * scale.view(1, -1, 1)).reshape(-1)
        flat[lo:lo + n] = x
    return out


def bits_from_device(t):
    """bfloat16 torch tensor -> uint16 numpy bit patterns (host)."""
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
