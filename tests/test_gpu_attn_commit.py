"""GPU parity of sdvg_block_attn_commit (attention with the block's commit fused into the same
launch) and sdvg_kv_commit_mark through the C ABI: the attention output is bit-identical to
sdvg_block_attn's and within the bounds against the oracle; the cache after the fused calls is
bit-identical to the oracle's mirror after oracle.kv_commit; nothing outside the slot changes."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import BF16_MAX_ABS, BF16_REL_RMS, attn_errors, bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu
CANARY = 0x7FC1


@pytest.mark.parametrize("L,H,T,n_cached,head_major", [(1, 12, 312, 2, False), (3, 2, 70, 1, False), (2, 3, 33, 0, True),
                                                       (2, 5, 257, 3, True)])
def test_fused_commit_small(L, H, T, n_cached, head_major):
    import paper_2604_17397_amd as P
    cap = (n_cached + 2) * T
    c_len = n_cached * T
    mirror = oracle.KVMirror(L, cap, H, 128, T, fill=CANARY)
    if head_major:
        k = torch.empty((L, H, cap, 128), dtype=torch.bfloat16, device="cuda").transpose(1, 2)
        v = torch.empty((L, H, cap, 128), dtype=torch.bfloat16, device="cuda").transpose(1, 2)
    else:
        k = torch.empty((L, cap, H, 128), dtype=torch.bfloat16, device="cuda")
        v = torch.empty((L, cap, H, 128), dtype=torch.bfloat16, device="cuda")
    k.view(torch.int16).fill_(np.int16(CANARY))
    v.view(torch.int16).fill_(np.int16(CANARY))
    cache = P.KVCache(k, v, T)
    for s in range(n_cached):       # fill the cached blocks through the ordinary commit
        bk = si.normal_bf16(600 + s, si.TID_K_BLK, (L, T, H, 128))
        bv = si.normal_bf16(600 + s, si.TID_V_BLK, (L, T, H, 128))
        assert oracle.kv_commit(mirror, bk, bv, s) == 0
        P.kv_commit(cache, to_dev_bf16(bk), to_dev_bf16(bv), s)
    q = si.normal_bf16(610, si.TID_Q, (T, H, 128))
    bk = si.normal_bf16(611, si.TID_K_BLK, (L, T, H, 128))
    bv = si.normal_bf16(611, si.TID_V_BLK, (L, T, H, 128))
    dq, dbk, dbv = to_dev_bf16(q), to_dev_bf16(bk), to_dev_bf16(bv)
    for l in range(L):
        kc, vc = cache.layer(l)
        plain = P.block_attn(dq, kc, vc, dbk[l], dbv[l], c_len)
        fused = P.block_attn_commit(dq, kc, vc, dbk[l], dbv[l], c_len)
        torch.cuda.synchronize()
        assert torch.equal(plain.view(torch.int16), fused.view(torch.int16))
        ref = oracle.block_attn(q, mirror.k[l], mirror.v[l], bk[l], bv[l], c_len)
        max_abs, rel = attn_errors(bits_of(fused), ref)
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS, (max_abs, rel)
    # the length only moves with the mark; the mark follows the append-only rule
    assert cache.cache_len == c_len
    with pytest.raises(P.SdvgError):
        P.kv_commit_mark(cache, n_cached + 1)
    P.kv_commit_mark(cache, n_cached)
    assert oracle.kv_commit(mirror, bk, bv, n_cached) == 0
    assert cache.cache_len == mirror.cache_len == c_len + T
    assert np.array_equal(bits_of(cache.k), mirror.k) and np.array_equal(bits_of(cache.v), mirror.v)


def test_fused_commit_rejects_bad_arguments():
    import paper_2604_17397_amd as P
    T, H = 64, 2
    k = torch.zeros((3 * T, H, 128), dtype=torch.bfloat16, device="cuda")
    q = torch.zeros((T, H, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(ValueError):
        P.block_attn_commit(q, k, k.clone(), q, q, 2 * T + 1)          # no room after cache_len
    with pytest.raises(P.SdvgError) as e:
        P.block_attn_commit(q, k, k.clone(), k[T:2 * T], q, T)          # the block IS the destination rows
    assert e.value.status == -3
    with pytest.raises(ValueError):
        P.block_attn_commit(q, None, None, q, q, 0)


def test_fused_commit_at_target_shape():
    # one layer at the headline shape: 40 heads, 6 cached blocks, the 7th slot filled by the launch
    import paper_2604_17397_amd as P
    T, H, nb = 4680, 40, 6
    c_len = nb * T
    k = si.device_normal_bf16(((nb + 1) * T, H, 128), 620, si.TID_K_CACHE)
    v = si.device_normal_bf16(((nb + 1) * T, H, 128), 620, si.TID_V_CACHE)
    k[c_len:].view(torch.int16).fill_(np.int16(CANARY))
    v[c_len:].view(torch.int16).fill_(np.int16(CANARY))
    q = si.device_normal_bf16((T, H, 128), 620, si.TID_Q)
    kb = si.device_normal_bf16((T, H, 128), 620, si.TID_K_BLK)
    vb = si.device_normal_bf16((T, H, 128), 620, si.TID_V_BLK)
    plain = P.block_attn(q, k, v, kb, vb, c_len)
    fused = P.block_attn_commit(q, k, v, kb, vb, c_len)
    torch.cuda.synchronize()
    assert torch.equal(plain.view(torch.int16), fused.view(torch.int16))
    assert torch.equal(k[c_len:].view(torch.int16), kb.view(torch.int16))
    assert torch.equal(v[c_len:].view(torch.int16), vb.view(torch.int16))
    rows = si.parity_rows(T)[::8]
    f = si.bits_from_device
    ref = oracle.block_attn(f(q), f(k[:c_len]), f(v[:c_len]), f(kb), f(vb), c_len, rows=rows)
    max_abs, rel = attn_errors(f(fused)[rows], ref)
    assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS, (max_abs, rel)
