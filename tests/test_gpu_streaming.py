"""Full 7-block streaming generation at drafter and target shapes (synthetic driver of the
paper's per-block loop, Sec. 3 "Inference flow"): for block k = 0..6, S = 4 denoising steps x
L layers of block attention with cache_len = 4680 k over a real [L][7T][H][128] cache, then the
router on seeded scores and commit (accept) or rollback + commit of the regenerated block
(reject). One layer per block is compared with the oracle on sampled rows, and two layers of the
final cache are compared with an oracle mirror that replayed the same commit/rollback sequence.
"""
import time

import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import BF16_MAX_ABS, BF16_REL_RMS, attn_errors

pytestmark = pytest.mark.gpu

T, NB, S, TAU = 4680, 7, 4, -0.7


@pytest.mark.parametrize("name", ["drafter", "target"])
def test_streaming_generation(name):
    import paper_2604_17397_amd as P
    cfg = si.CONFIGS[name]
    L, H = cfg["n_layers"], cfg["n_heads"]
    f = si.bits_from_device
    k = torch.zeros((L, NB * T, H, 128), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros_like(k)
    cache = P.KVCache(k, v, T)
    mirror_layers = [0, L - 1]
    mirrors = {l: oracle.KVMirror(1, NB * T, H, 128, T) for l in mirror_layers}
    q = si.device_normal_bf16((T, H, 128), 400, si.TID_Q)
    out = torch.empty_like(q)
    scores = si.frame_scores_correlated(401, NB)
    heads = [0, H // 3, H - 1]
    rows = si.parity_rows(T)[::4]
    flops, attn_ms, accepted = 0.0, 0.0, 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for b in range(NB):
        c_len = b * T
        assert cache.cache_len == c_len
        draft_k = si.device_normal_bf16((L, T, H, 128), 410 + b, si.TID_K_BLK)
        draft_v = si.device_normal_bf16((L, T, H, 128), 410 + b, si.TID_V_BLK)
        e0.record()
        for _ in range(S):
            for l in range(L):
                kc, vc = cache.layer(l)
                P.block_attn(q, kc, vc, draft_k[l], draft_v[l], c_len, out=out)
        e1.record()
        torch.cuda.synchronize()
        attn_ms += e0.elapsed_time(e1)
        flops += S * L * si.attn_flops(T, c_len + T, H)
        # parity of one layer of this block on the row sample
        l = b % L
        kc, vc = cache.layer(l)
        P.block_attn(q, kc, vc, draft_k[l], draft_v[l], c_len, out=out)
        torch.cuda.synchronize()
        ref = oracle.block_attn(f(q[:, heads]), f(kc[:max(c_len, 1), heads]), f(vc[:max(c_len, 1), heads]),
                                f(draft_k[l][:, heads]), f(draft_v[l][:, heads]), c_len, rows=rows)
        max_abs, rel = attn_errors(f(out[:, heads])[rows], ref)
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS, (b, max_abs, rel)
        # stage the draft, route, keep it or replace it by the regenerated block
        P.kv_commit(cache, draft_k, draft_v, b)
        for ml in mirror_layers:
            assert oracle.kv_commit(mirrors[ml], f(draft_k[ml])[None], f(draft_v[ml])[None], b) == 0
        dec, qb = P.worst_frame_route(torch.from_numpy(scores[b]).cuda(), TAU, b)
        want = oracle.route(scores[b], TAU, b)
        assert dec == want[0] and qb.view(np.uint32) == want[1].view(np.uint32)
        if b == 0:
            assert dec == 0   # block 0 is always regenerated
        if dec:
            accepted += 1
        else:
            P.kv_rollback(cache, c_len)
            regen_k = si.device_normal_bf16((L, T, H, 128), 430 + b, si.TID_K_BLK)
            regen_v = si.device_normal_bf16((L, T, H, 128), 430 + b, si.TID_V_BLK)
            P.kv_commit(cache, regen_k, regen_v, b)
            for ml in mirror_layers:
                assert oracle.kv_rollback(mirrors[ml], c_len) == 0
                assert oracle.kv_commit(mirrors[ml], f(regen_k[ml])[None], f(regen_v[ml])[None], b) == 0
            del regen_k, regen_v
        del draft_k, draft_v
    torch.cuda.synchronize()
    assert cache.cache_len == NB * T
    for ml in mirror_layers:
        assert mirrors[ml].cache_len == NB * T
        assert np.array_equal(f(k[ml]), mirrors[ml].k[0]) and np.array_equal(f(v[ml]), mirrors[ml].v[0])
    print("\n%s streaming: %.1f TFLOP of attention in %.1f ms = %.1f TFLOP/s aggregate; accepted %d of %d blocks"
          % (name, flops / 1e12, attn_ms, flops / attn_ms / 1e9, accepted, NB))
