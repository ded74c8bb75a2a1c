"""The asynchronous entry points on a side stream and recorded into a HIP graph: every replay
is checked against the eager result."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu


def test_side_stream_and_graph_replay():
    """The asynchronous calls run on the caller's stream and can be captured into a HIP graph:
    attention + commit + batched routing + rollback recorded once on a side stream, replayed
    three times with eager work in between; every replay must reproduce the eager results."""
    import paper_2604_17397_amd as P
    H, T, c_len, L = 2, 72, 144, 2
    q, kc, vc, kb, vb = si.attn_inputs(H, T, c_len, seed=77, cache_capacity=c_len + T)
    dq, dkb, dvb = to_dev_bf16(q), to_dev_bf16(kb), to_dev_bf16(vb)
    k = torch.zeros((L, c_len + T, H, 128), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros_like(k)
    k[0, :c_len], v[0, :c_len] = to_dev_bf16(kc[:c_len]), to_dev_bf16(vc[:c_len])
    blk_k = torch.stack([dkb, dkb]).contiguous()
    blk_v = torch.stack([dvb, dvb]).contiguous()
    scores = torch.from_numpy(si.frame_scores_correlated(5, 8)).cuda()
    cache = P.KVCache(k, v, T, cache_len=c_len)
    out = torch.empty_like(dq)

    def work(cache_len_before):
        cache.c.cache_len = cache_len_before   # the host field is not part of a replay
        P.block_attn(dq, k[0], v[0], dkb, dvb, c_len, out=out)
        P.kv_commit(cache, blk_k, blk_v, c_len // T)
        dec, qb = P.worst_frame_route_batch(scores, -0.7, first_block_idx=0)
        snap = k.clone()
        P.kv_rollback(cache, c_len)
        return dec, qb, snap

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dec_e, qb_e, snap_e = work(c_len)      # eager on the side stream (also warms up)
        side.synchronize()
        out_e, k_e = out.clone(), k.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            dec_g, qb_g, snap_g = work(c_len)
        for rep in range(3):
            out.zero_()
            k[:, c_len:].fill_(1.0)            # eager work between replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), out_e.view(torch.int16)), rep
            assert torch.equal(dec_g, dec_e) and torch.equal(qb_g.view(torch.int32), qb_e.view(torch.int32))
            assert torch.equal(snap_g.view(torch.int16), snap_e.view(torch.int16))
            assert torch.equal(k.view(torch.int16), k_e.view(torch.int16))
    ref = oracle.block_attn(q, kc[:c_len], vc[:c_len], kb, vb, c_len)
    from gpu_util import attn_errors, BF16_MAX_ABS
    assert attn_errors(bits_of(out_e), ref)[0] <= BF16_MAX_ABS
    assert snap_e[0, c_len:].abs().sum().item() > 0 and k_e[:, c_len:].abs().sum().item() == 0
