"""sdvg_block_attn_batch_static, the entry point that allocates nothing (its key-split workspace
is a fixed array inside the library): through the C ABI, two calls in a row -- the second with a
smaller input, so that stale partial results of the first call lie in the array -- each checked
against sdvg_block_attn_batch with a caller workspace (same kernels, same plan: bit-identical)
and against the oracle; a shape whose split exceeds the array is rejected on the host."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import BF16_MAX_ABS, BF16_REL_RMS, attn_errors

pytestmark = pytest.mark.gpu

T = 4680


def case(P, H, n_q, c_len, seed):
    q = si.device_normal_bf16((n_q, H, 128), seed, si.TID_Q)
    kb = si.device_normal_bf16((n_q, H, 128), seed, si.TID_K_BLK)
    vb = si.device_normal_bf16((n_q, H, 128), seed, si.TID_V_BLK)
    kc = si.device_normal_bf16((c_len, H, 128), seed, si.TID_K_CACHE)
    vc = si.device_normal_bf16((c_len, H, 128), seed, si.TID_V_CACHE)
    need = P.block_attn_workspace_bytes(q, kc, vc, kb, vb, c_len, split="always")
    assert 0 < need <= P.lib().sdvg_block_attn_static_workspace_limit()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    want = P.block_attn_batch([q], [kc], [vc], [kb], [vb], c_len, workspace=ws, split="always")[0]
    got = torch.full_like(q, float("nan"))                       # the caller still owns the output
    P.block_attn_batch_static([q], [kc], [vc], [kb], [vb], c_len, outs=[got], split="always")
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    rows = si.parity_rows(n_q)[::5]
    f = si.bits_from_device
    ref = oracle.block_attn(f(q), f(kc), f(vc), f(kb), f(vb), c_len, rows=rows)
    max_abs, rel = attn_errors(f(got)[rows], ref)
    assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_RMS, (max_abs, rel)


def test_static_workspace_two_calls_second_smaller():
    import paper_2604_17397_amd as P
    case(P, H=2, n_q=T, c_len=6 * T, seed=501)     # 38 query tiles over 256 workgroups, 294 partial slots
    case(P, H=1, n_q=T, c_len=2 * T, seed=502)     # 19 query tiles, shorter key range, fewer slots


def test_static_workspace_rejects_what_does_not_fit():
    import paper_2604_17397_amd as P
    H, c_len = 40, T
    q = si.device_normal_bf16((T, H, 128), 3, si.TID_Q)
    kv = si.device_normal_bf16((c_len, H, 128), 3, si.TID_K_CACHE)
    need = P.block_attn_workspace_bytes(q, kv, kv, q, q, c_len, split="always")
    assert need > P.lib().sdvg_block_attn_static_workspace_limit()
    out = torch.zeros_like(q)
    with pytest.raises(P.SdvgError) as e:
        P.block_attn_batch_static([q], [kv], [kv], [q], [q], c_len, outs=[out], split="always")
    assert e.value.status == -3
    torch.cuda.synchronize()
    assert out.abs().sum().item() == 0                              # nothing was launched
    # without a split the same shape runs (no workspace needed)
    P.block_attn_batch_static([q], [kv], [kv], [q], [q], c_len, outs=[out], split="never")
    torch.cuda.synchronize()
    assert out.abs().sum().item() > 0
