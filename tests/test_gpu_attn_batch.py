"""GPU parity of sdvg_block_attn_batch through the C ABI: several (q, cache, block, out) sets in
one launch (the conditional and unconditional pass of classifier-free guidance, Sec. 4.1 "Models")
and the key split with its merge kernel. The oracle is the plain definition applied to every
item on its own; the unsplit single-item call is the second reference."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import BF16_MAX_ABS, BF16_REL_RMS, attn_errors, attn_errors_by_head, bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu


def make_items(n_items, H, n_q, c_len, seed, jitter=False):
    items = []
    for i in range(n_items):
        q, kc, vc, kb, vb = si.attn_inputs(H, n_q, c_len, seed=seed + 10 * i, jitter=jitter,
                                           cache_capacity=max(c_len, 1))
        items.append(dict(q=q, kc=kc, vc=vc, kb=kb, vb=vb))
    return items


def run_batch(P, items, c_len, workspace=None):
    dev = [dict((k, to_dev_bf16(v)) for k, v in it.items()) for it in items]
    outs = [torch.full_like(d["q"], float("nan")) for d in dev]
    P.block_attn_batch([d["q"] for d in dev], [d["kc"] for d in dev] if c_len else None,
                       [d["vc"] for d in dev] if c_len else None, [d["kb"] for d in dev], [d["vb"] for d in dev],
                       c_len, outs=outs, workspace=workspace)
    torch.cuda.synchronize()
    return dev, outs


@pytest.mark.parametrize("n_items,H,n_q,c_len", [(2, 12, 312, 624), (1, 3, 70, 0), (3, 2, 333, 100), (8, 1, 40, 65),
                                                 (2, 5, 257, 4680)])
def test_batch_matches_oracle_item_by_item(n_items, H, n_q, c_len):
    import paper_2604_17397_amd as P
    items = make_items(n_items, H, n_q, c_len, seed=300 + n_items)
    dev, outs = run_batch(P, items, c_len)
    for it, d, o in zip(items, dev, outs):
        ref = oracle.block_attn(it["q"], it["kc"], it["vc"], it["kb"], it["vb"], c_len)
        max_abs, rel = attn_errors(bits_of(o), ref)
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS, (max_abs, rel)
        # and bit-identical to the single-item entry point (same kernel, same order of operations)
        single = P.block_attn(d["q"], d["kc"] if c_len else None, d["vc"] if c_len else None, d["kb"], d["vb"], c_len)
        assert torch.equal(single.view(torch.int16), o.view(torch.int16))


def test_batch_rejects_bad_arguments():
    import paper_2604_17397_amd as P
    items = make_items(2, 2, 40, 64, seed=5)
    dev = [dict((k, to_dev_bf16(v)) for k, v in it.items()) for it in items]
    qs, kcs, vcs = [d["q"] for d in dev], [d["kc"] for d in dev], [d["vc"] for d in dev]
    kbs, vbs = [d["kb"] for d in dev], [d["vb"] for d in dev]
    with pytest.raises(P.SdvgError):
        P.block_attn_batch(qs * 5, kcs * 5, vcs * 5, kbs * 5, vbs * 5, 64)     # 10 items > 8
    with pytest.raises(ValueError):
        P.block_attn_batch(qs, kcs, vcs, [kbs[0], kbs[1][:30]], [vbs[0], vbs[1][:30]], 64)   # shapes differ
    with pytest.raises(ValueError):
        P.block_attn_batch(qs, kcs, vcs, kbs, vbs, 65)                         # longer than the cache


def close_ulps(a, b):
    """Split and unsplit runs round P to bf16 against different running maxima and add in a
    different order, so they are two roundings of the same numbers: the difference stays within
    the error each of them is allowed against the oracle."""
    a, b = a.double(), b.double()
    d = a - b
    return bool(d.abs().max() <= BF16_MAX_ABS and (d * d).sum().sqrt() <= 0.5 * BF16_REL_RMS * (a * a).sum().sqrt())


def split_shape_case(P, n_items, H, T, c_len, seed, jitter, split="always"):
    """Runs a shape for which the library splits keys (checked via the workspace query), with and
    without the workspace; returns device tensors, outputs and host bits for the oracle."""
    hs = [si.head_scales(seed, H, w) for w in range(3)] if jitter else [None] * 3
    dev = []
    for i in range(n_items):
        s = seed + 7 * i
        dev.append(dict(q=si.device_normal_bf16((T, H, 128), s, si.TID_Q, head_scale=hs[0]),
                        kb=si.device_normal_bf16((T, H, 128), s, si.TID_K_BLK, head_scale=hs[1]),
                        vb=si.device_normal_bf16((T, H, 128), s, si.TID_V_BLK, head_scale=hs[2]),
                        kc=si.device_normal_bf16((c_len, H, 128), s, si.TID_K_CACHE, head_scale=hs[1]),
                        vc=si.device_normal_bf16((c_len, H, 128), s, si.TID_V_CACHE, head_scale=hs[2])))
    d0 = dev[0]
    need = P.block_attn_workspace_bytes(d0["q"], d0["kc"], d0["vc"], d0["kb"], d0["vb"], c_len, n_items=n_items,
                                        split=split)
    assert need > 0, "the library is expected to split keys for this shape"
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    args = ([d["q"] for d in dev], [d["kc"] for d in dev], [d["vc"] for d in dev], [d["kb"] for d in dev],
            [d["vb"] for d in dev], c_len)
    plain = P.block_attn_batch(*args)
    split = P.block_attn_batch(*args, outs=[torch.full_like(d["q"], float("nan")) for d in dev], workspace=ws,
                               split=split)
    torch.cuda.synchronize()
    return dev, plain, split


def test_key_split_at_drafter_shape():
    # 12 heads x 19 query tiles = 228 workgroups for 256 compute units: the keys (2 cached blocks
    # + the block = 14040) are dealt out over 256 workgroups and merged. Per-head jitter.
    import paper_2604_17397_amd as P
    T, H, c_len = 4680, 12, 2 * 4680
    dev, plain, split = split_shape_case(P, 1, H, T, c_len, seed=401, jitter=True)
    assert not torch.isnan(split[0].float()).any()
    rows = si.parity_rows(T)
    f = si.bits_from_device
    d = dev[0]
    ref = oracle.block_attn(f(d["q"]), f(d["kc"]), f(d["vc"]), f(d["kb"]), f(d["vb"]), c_len, rows=rows)
    for name, o in (("plain", plain[0]), ("split", split[0])):
        max_abs, rel, worst, head = attn_errors_by_head(f(o)[rows], ref)
        print("%s: max|err| %.3e rel-RMS %.3e worst head %d %.3e" % (name, max_abs, rel, head, worst))
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS and worst <= BF16_REL_RMS
    assert close_ulps(plain[0], split[0])


def test_key_split_two_items_small_cache():
    # cond + uncond at the drafter shape: 456 query tiles = 1.78 rounds -> split over 512 workgroups.
    # A short cache (1 block) makes pieces that start and end near the seam.
    import paper_2604_17397_amd as P
    T, H, c_len = 4680, 12, 4680
    dev, plain, split = split_shape_case(P, 2, H, T, c_len, seed=402, jitter=False)
    rows = si.parity_rows(T)[::4]
    f = si.bits_from_device
    for d, o in zip(dev, split):
        assert not torch.isnan(o.float()).any()
        ref = oracle.block_attn(f(d["q"]), f(d["kc"]), f(d["vc"]), f(d["kb"]), f(d["vb"]), c_len, rows=rows)
        max_abs, rel = attn_errors(f(o)[rows], ref)
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS, (max_abs, rel)
    for a, b in zip(plain, split):
        assert close_ulps(a, b)


def test_auto_policy_splits_few_heads_but_not_the_drafter_shape():
    # 5 heads x 19 query tiles = 95 workgroups for 256 compute units: AUTO splits; the 12-head
    # drafter layer (228 workgroups, 11 % idle) is left alone because the split costs more.
    import paper_2604_17397_amd as P
    T, c_len = 4680, 2 * 4680
    dev, plain, split = split_shape_case(P, 1, 5, T, c_len, seed=403, jitter=True, split="auto")
    rows = si.parity_rows(T)[::2]
    f = si.bits_from_device
    d = dev[0]
    ref = oracle.block_attn(f(d["q"]), f(d["kc"]), f(d["vc"]), f(d["kb"]), f(d["vb"]), c_len, rows=rows)
    max_abs, rel = attn_errors(f(split[0])[rows], ref)
    assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS, (max_abs, rel)
    assert close_ulps(plain[0], split[0])
    q12 = si.device_normal_bf16((T, 12, 128), 1, si.TID_Q)
    kv12 = si.device_normal_bf16((c_len, 12, 128), 1, si.TID_K_CACHE)
    assert P.block_attn_workspace_bytes(q12, kv12, kv12, q12, q12, c_len, split="auto") == 0
    assert P.block_attn_workspace_bytes(q12, kv12, kv12, q12, q12, c_len, split="always") > 0
    assert P.block_attn_workspace_bytes(q12, kv12, kv12, q12, q12, c_len, split="never") == 0


def test_small_workspace_falls_back_to_the_plain_launch():
    import paper_2604_17397_amd as P
    T, H, c_len = 4680, 12, 4680
    q = si.device_normal_bf16((T, H, 128), 9, si.TID_Q)
    kb = si.device_normal_bf16((T, H, 128), 9, si.TID_K_BLK)
    vb = si.device_normal_bf16((T, H, 128), 9, si.TID_V_BLK)
    kc = si.device_normal_bf16((c_len, H, 128), 9, si.TID_K_CACHE)
    vc = si.device_normal_bf16((c_len, H, 128), 9, si.TID_V_CACHE)
    ws = torch.empty(4096, dtype=torch.uint8, device="cuda")
    a = P.block_attn_batch([q], [kc], [vc], [kb], [vb], c_len, workspace=ws, split="always")[0]
    b = P.block_attn(q, kc, vc, kb, vb, c_len)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
