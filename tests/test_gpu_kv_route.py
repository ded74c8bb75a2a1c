"""GPU parity, bit-exact: sdvg_kv_commit / sdvg_kv_rollback / sdvg_worst_frame_route(_batch)
through the C ABI against the CPU oracle."""
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

def gpu_route(P, scores, tau, b):
    return P.worst_frame_route(torch.from_numpy(np.asarray(scores, np.float32)).cuda(), tau, b)


def same_route(a, b):
    return a[0] == b[0] and np.float32(a[1]).view(np.uint32) == np.float32(b[1]).view(np.uint32)


def test_tiny_config_route():
    import paper_2604_17397_amd as P
    scores = si.normal(si.SEED, si.TID_SCORES, 12).astype(np.float32)
    for b in (0, 1):
        assert same_route(gpu_route(P, scores, -0.7, b), oracle.route(scores, -0.7, b))
    assert gpu_route(P, scores, -0.7, 0)[0] == 0


@pytest.mark.parametrize("F", [1, 3, 9, 12, 63, 64, 65, 200])
def test_route_frame_counts(F):
    import paper_2604_17397_amd as P
    for trial in range(4):
        s = si.frame_scores_iid(50 + trial, 1, n_frames=F)[0]
        for tau in (-1.0, -0.7, -0.4, float(s.min())):
            assert same_route(gpu_route(P, s, tau, 3), oracle.route(s, tau, 3))


def test_route_edge_values():
    import paper_2604_17397_amd as P
    cases = [[0.0, -0.0, 1.0], [-0.0, 0.0], [1.0, 0.0, -0.0], [np.inf] * 12, [-np.inf, 1.0],
             [0.2, np.nan, 0.1], [np.nan], [np.inf, -np.inf, np.nan], [1e-45, -1e-45], [3.0]]
    for c in cases:
        for tau in (0.0, -0.0, -0.7, np.inf, -np.inf):
            for b in (0, 2):
                assert same_route(gpu_route(P, c, tau, b), oracle.route(c, tau, b)), (c, tau, b)


def test_route_batch_matches_oracle_for_both_score_generators():
    import paper_2604_17397_amd as P
    n = 4096
    for gen in (si.frame_scores_iid, si.frame_scores_correlated):
        scores = gen(77, n)
        idx = (np.arange(n) % 9).astype(np.int32)
        for tau in (-1.0, -0.7, -0.4):
            dec, qb = P.worst_frame_route_batch(torch.from_numpy(scores).cuda(), tau,
                                                block_idx=torch.from_numpy(idx).cuda())
            dec, qb = dec.cpu().numpy(), qb.cpu().numpy()
            for i in range(n):
                d, q = oracle.route(scores[i], tau, int(idx[i]))
                assert d == dec[i] and q.view(np.uint32) == qb[i].view(np.uint32)
            assert dec[idx == 0].sum() == 0
        dec2, _ = P.worst_frame_route_batch(torch.from_numpy(scores).cuda(), -0.7, first_block_idx=0)
        assert dec2[0].item() == 0


def test_avg_frame_route_matches_oracle():
    """The ablation's average-frame router (fp64 sum in frame order), bit-exact, single and batched."""
    import paper_2604_17397_amd as P

    def gpu(scores, tau, b):
        return P.worst_frame_route(torch.from_numpy(np.asarray(scores, np.float32)).cuda(), tau, b, mode="mean")

    for F in (1, 3, 12, 65, 200):
        for trial in range(3):
            s = si.frame_scores_iid(90 + trial, 1, n_frames=F)[0]
            for tau in (-0.5, -0.3, float(np.float32(s.astype(np.float64).mean()))):
                for b in (0, 4):
                    assert same_route(gpu(s, tau, b), oracle.route(s, tau, b, mode="mean")), (F, tau, b)
    cases = [[16777216.0, 1.0, 1.0, -16777216.0], [0.5, 0.25, 0.25], [np.inf, 1.0], [np.inf, -np.inf],
             [0.2, np.nan, 0.1], [-0.0, -0.0], [1e-45, 1e-45, 0.0], [3.4e38, 3.4e38]]
    for c in cases:
        for tau in (0.0, 0.5, -np.inf):
            assert same_route(gpu(c, tau, 2), oracle.route(np.array(c, np.float32), tau, 2, mode="mean")), (c, tau)
    n = 2048
    scores = si.frame_scores_correlated(78, n)
    idx = (np.arange(n) % 9).astype(np.int32)
    for tau in (-0.5, -0.3):
        dec, qb = P.worst_frame_route_batch(torch.from_numpy(scores).cuda(), tau,
                                            block_idx=torch.from_numpy(idx).cuda(), mode="mean")
        dec, qb = dec.cpu().numpy(), qb.cpu().numpy()
        for i in range(n):
            d, q = oracle.route(scores[i], tau, int(idx[i]), mode="mean")
            assert d == dec[i] and q.view(np.uint32) == qb[i].view(np.uint32)
        assert dec[idx == 0].sum() == 0


@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 4096 + 5, (64 << 20) + 3])
def test_buffer_snapshot_matches_oracle(n):
    """Snapshot / restore of an opaque buffer: bit-exact, margins untouched, round trip."""
    import paper_2604_17397_amd as P
    g = torch.Generator(device="cuda")
    g.manual_seed(1234 + n % 97)
    src = torch.randint(0, 256, (n + 32,), dtype=torch.uint8, device="cuda", generator=g)
    dst = torch.full((n + 48,), 0xA5, dtype=torch.uint8, device="cuda")
    h_dst = dst.cpu().numpy().copy()
    oracle.buffer_copy(h_dst, src.cpu().numpy(), n)
    P.buffer_snapshot(dst, src, n)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy(), h_dst)
    # clone -> corrupt -> restore
    live = src[:n].clone() if n else src[:0].clone()
    snap = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
    P.buffer_snapshot(snap, live, n)
    orig = live.cpu().numpy().copy()
    if n:
        live[::3] ^= 0xFF
    P.buffer_snapshot(live, snap, n)
    torch.cuda.synchronize()
    assert np.array_equal(live.cpu().numpy(), orig)


def test_mfma_probe_runs():
    """The MFMA-only measurement kernel: runs, reports its FLOP count and a clock reading."""
    import paper_2604_17397_amd as P
    flops, cycles = P.probe_mfma(500)
    torch.cuda.synchronize()
    assert flops == 256 * 4 * 500 * 16 * 32768.0
    assert int(cycles.item()) > 500 * 16 * 8   # at least a quarter of the MFMA-bound cycle count
    with pytest.raises(P.SdvgError):
        P.probe_mfma(0)


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
