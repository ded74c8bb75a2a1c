"""GPU parity, bit-exact: sdvg_rope and sdvg_kv_commit_rope through the C ABI against the oracle's
rotary embedding (same fp32 operations in the same order on both sides, so the bf16 results must
be identical), and the property that makes RoPE worth having: attention over rotated q / k depends
on relative positions only."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import BF16_MAX_ABS, BF16_REL_RMS, attn_errors, bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu
CANARY = 0x7FC1


def angle_tables(n_tokens, first_pos=0.0, seed=None):
    """cos / sin float32 [n_tokens, 64]: 1-D positions first_pos + t with the usual geometric
    frequencies, or random angles when a seed is given."""
    if seed is None:
        theta = 10000.0 ** (-np.arange(64) / 64.0)
        ang = (first_pos + np.arange(n_tokens))[:, None] * theta[None, :]
    else:
        ang = np.random.default_rng(seed).uniform(-100, 100, (n_tokens, 64))
    return np.cos(ang).astype(np.float32), np.sin(ang).astype(np.float32)


@pytest.mark.parametrize("n,H", [(1, 1), (7, 3), (312, 12), (1031, 5), (4680, 40)])
def test_rope_bit_exact(n, H):
    import paper_2604_17397_amd as P
    if n * H > 100000:
        x = si.bits_from_device(si.device_normal_bf16((n, H, 128), 800, si.TID_Q))
    else:
        x = si.normal_bf16(800 + n, 0, (n, H, 128))
    c, s = angle_tables(n, seed=n)
    want = oracle.rope(x, c, s)
    dx, dc, ds = to_dev_bf16(x), torch.from_numpy(c).cuda(), torch.from_numpy(s).cuda()
    got = P.rope(dx, dc, ds)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(got), want)
    # in place, and through a strided (head-major) view
    y = dx.clone()
    P.rope(y, dc, ds, out=y)
    hm = dx.transpose(0, 1).contiguous().transpose(0, 1)            # [n, H, 128] with head-major strides
    got_hm = P.rope(hm, dc, ds, out=torch.empty_like(hm))
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(y), want) and np.array_equal(bits_of(got_hm), want)


def test_rope_rejects_bad_arguments():
    import paper_2604_17397_amd as P
    x = torch.zeros((8, 2, 128), dtype=torch.bfloat16, device="cuda")
    c = torch.ones((8, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(ValueError):
        P.rope(x, c[:7], c)
    with pytest.raises(ValueError):
        P.rope(x[:, :, :64], c, c)
    with pytest.raises(ValueError):
        P.rope(x, c.double(), c)


@pytest.mark.parametrize("L,H,T,head_major", [(1, 12, 312, False), (3, 2, 33, True), (2, 5, 1031, False)])
def test_commit_rope_bit_exact(L, H, T, head_major):
    import paper_2604_17397_amd as P
    cap = 3 * T
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
    for slot in range(2):
        bk = si.normal_bf16(810 + slot, si.TID_K_BLK, (L, T, H, 128))
        bv = si.normal_bf16(810 + slot, si.TID_V_BLK, (L, T, H, 128))
        c, s = angle_tables(T, first_pos=slot * T)
        rotated = np.stack([oracle.rope(bk[l], c, s) for l in range(L)])
        assert oracle.kv_commit(mirror, rotated, bv, slot) == 0          # oracle: rotate, then the plain commit
        P.kv_commit_rope(cache, to_dev_bf16(bk), to_dev_bf16(bv), slot, torch.from_numpy(c).cuda(),
                         torch.from_numpy(s).cuda())
        torch.cuda.synchronize()
        assert cache.cache_len == mirror.cache_len == (slot + 1) * T
        assert np.array_equal(bits_of(cache.k), mirror.k) and np.array_equal(bits_of(cache.v), mirror.v)
    with pytest.raises(P.SdvgError):     # append-only, like the plain commit
        P.kv_commit_rope(cache, to_dev_bf16(bk), to_dev_bf16(bv), 0, torch.from_numpy(c).cuda(), torch.from_numpy(s).cuda())


def test_attention_over_rotated_keys_sees_relative_positions_only():
    """Two runs of the same block attention whose positions differ by a common offset of 1000:
    q and k are rotated with sdvg_rope / sdvg_kv_commit_rope, attention by sdvg_block_attn. The
    outputs agree up to the rounding of the rotated rows; each also matches the oracle run on the
    oracle's own rotated rows."""
    import paper_2604_17397_amd as P
    H, T = 4, 200
    q = si.normal_bf16(820, si.TID_Q, (T, H, 128))
    bk = si.normal_bf16(820, si.TID_K_BLK, (1, T, H, 128))
    bv = si.normal_bf16(820, si.TID_V_BLK, (1, T, H, 128))
    ck = si.normal_bf16(821, si.TID_K_BLK, (1, T, H, 128))
    cv = si.normal_bf16(821, si.TID_V_BLK, (1, T, H, 128))
    outs = []
    for offset in (0.0, 1000.0):
        k = torch.zeros((1, 2 * T, H, 128), dtype=torch.bfloat16, device="cuda")
        v = torch.zeros_like(k)
        cache = P.KVCache(k, v, T)
        tab0, tab1 = angle_tables(T, offset), angle_tables(T, offset + T)
        dev = lambda t: torch.from_numpy(t).cuda()
        P.kv_commit_rope(cache, to_dev_bf16(ck), to_dev_bf16(cv), 0, dev(tab0[0]), dev(tab0[1]))   # cached block
        rq = P.rope(to_dev_bf16(q), dev(tab1[0]), dev(tab1[1]))                                    # current block
        rk = P.rope(to_dev_bf16(bk[0]), dev(tab1[0]), dev(tab1[1]))
        out = P.block_attn(rq, k[0], v[0], rk, to_dev_bf16(bv[0]), T)
        torch.cuda.synchronize()
        ref = oracle.block_attn(oracle.rope(q, *tab1), oracle.rope(ck[0], *tab0), cv[0], oracle.rope(bk[0], *tab1),
                                bv[0], T)
        max_abs, rel = attn_errors(bits_of(out), ref)
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS, (offset, max_abs, rel)
        outs.append(si.bf16_bits_to_f64(bits_of(out)))
    d = outs[0] - outs[1]
    assert np.sqrt((d * d).sum() / (outs[0] * outs[0]).sum()) <= 2 * BF16_REL_RMS
