"""GPU parity, bit-exact: sdvg_kv_commit / sdvg_kv_rollback through the C ABI against the CPU
oracle's host mirror of the cache."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu

CANARY = 0x7FC1  # NaN bit pattern


def make_pair(L, cap, H, T, head_major=False):
    import paper_2604_17397_amd as P
    m = oracle.KVMirror(L, cap, H, 128, T, fill=CANARY)
    if head_major:
        k = torch.empty((L, H, cap, 128), dtype=torch.bfloat16, device="cuda").transpose(1, 2)
        v = torch.empty((L, H, cap, 128), dtype=torch.bfloat16, device="cuda").transpose(1, 2)
    else:
        k = torch.empty((L, cap, H, 128), dtype=torch.bfloat16, device="cuda")
        v = torch.empty((L, cap, H, 128), dtype=torch.bfloat16, device="cuda")
    k.view(torch.int16).fill_(np.int16(CANARY))
    v.view(torch.int16).fill_(np.int16(CANARY))
    return P, m, P.KVCache(k, v, T)


def same(cache, m):
    torch.cuda.synchronize()
    gk = cache.k.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    gv = cache.v.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return cache.cache_len == m.cache_len and np.array_equal(gk, m.k) and np.array_equal(gv, m.v)


def block(seed, L, T, H):
    k = si.normal_bf16(seed, si.TID_K_BLK, (L * T, H, 128)).reshape(L, T, H, 128)
    v = si.normal_bf16(seed, si.TID_V_BLK, (L * T, H, 128)).reshape(L, T, H, 128)
    return k, v


@pytest.mark.parametrize("head_major", [False, True])
def test_tiny_config_commit_then_rollback(head_major):
    # tiny config: 12 heads, T = 312, two cached blocks, commit into slot 2, roll back to 624
    L, H, T, cap = 1, 12, 312, 4 * 312
    P, m, cache = make_pair(L, cap, H, T, head_major)
    for s in range(3):
        k, v = block(10 + s, L, T, H)
        assert oracle.kv_commit(m, k, v, s) == 0
        P.kv_commit(cache, to_dev_bf16(k), to_dev_bf16(v), s)
        assert same(cache, m)
    assert cache.cache_len == 936
    oracle.kv_rollback(m, 624)
    P.kv_rollback(cache, 624)
    assert cache.cache_len == 624 and same(cache, m)
    # rollback to the same length is a no-op; slot 2 can be refilled with other data
    P.kv_rollback(cache, 624)
    assert same(cache, m)
    k, v = block(99, L, T, H)
    oracle.kv_commit(m, k, v, 2)
    P.kv_commit(cache, to_dev_bf16(k), to_dev_bf16(v), 2)
    assert same(cache, m)


@pytest.mark.parametrize("L,H,T", [(3, 2, 5), (2, 5, 33), (4, 1, 1), (2, 3, 1031)])
def test_multi_layer_ragged_sizes_and_partial_rollback(L, H, T):
    cap = 3 * T + 2
    P, m, cache = make_pair(L, cap, H, T)
    for s in range(3):
        k, v = block(20 + s, L, T, H)
        oracle.kv_commit(m, k, v, s)
        P.kv_commit(cache, to_dev_bf16(k), to_dev_bf16(v), s)
    assert same(cache, m)
    new_len = T + T // 2
    oracle.kv_rollback(m, new_len)
    P.kv_rollback(cache, new_len)
    assert same(cache, m)
    oracle.kv_rollback(m, 0)
    P.kv_rollback(cache, 0)
    assert same(cache, m) and cache.cache_len == 0


def test_errors_leave_device_state_untouched():
    P, m, cache = make_pair(2, 16, 2, 4)
    k, v = block(1, 2, 4, 2)
    dk, dv = to_dev_bf16(k), to_dev_bf16(v)
    with pytest.raises(P.SdvgError) as e:
        P.kv_commit(cache, dk, dv, 1)
    assert e.value.status == -3
    with pytest.raises(P.SdvgError):
        P.kv_rollback(cache, 1)
    assert same(cache, m)


def test_attention_reads_what_commit_wrote():
    # end-to-end on the tiny config: commit two blocks, attend with cache_len = 624 through the
    # cache's layer view, compare with the oracle on the same bits
    from gpu_util import attn_errors, BF16_MAX_ABS, BF16_REL_RMS
    L, H, T = 2, 12, 312
    P, m, cache = make_pair(L, 3 * T, H, T)
    for s in range(2):
        k, v = block(30 + s, L, T, H)
        oracle.kv_commit(m, k, v, s)
        P.kv_commit(cache, to_dev_bf16(k), to_dev_bf16(v), s)
    q, _, _, kb, vb = si.attn_inputs(H, T, 0, seed=31)
    for layer in range(L):
        kc, vc = cache.layer(layer)
        out = P.block_attn(to_dev_bf16(q), kc, vc, to_dev_bf16(kb), to_dev_bf16(vb), cache.cache_len)
        torch.cuda.synchronize()
        ref = oracle.block_attn(q, m.k[layer], m.v[layer], kb, vb, m.cache_len)
        max_abs, rel = attn_errors(bits_of(out), ref)
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS


# ------------------------------------------------------------------ routing
