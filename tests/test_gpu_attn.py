"""GPU parity: sdvg_block_attn (through the C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si
from gpu_util import BF16_MAX_ABS, BF16_REL_RMS, attn_errors, bits_of, to_dev_bf16

pytestmark = pytest.mark.gpu


def run_case(H, n_blk, cache_len, seed=si.SEED, jitter=False, cap_extra=0, rows=None, n_q=None):
    import paper_2604_17397_amd as P
    q, kc, vc, kb, vb = si.attn_inputs(H, n_blk, cache_len, seed=seed, jitter=jitter,
                                       cache_capacity=cache_len + cap_extra)
    if n_q is not None:
        q = np.ascontiguousarray(q[:n_q])
    dq, dkb, dvb = to_dev_bf16(q), to_dev_bf16(kb), to_dev_bf16(vb)
    dkc = to_dev_bf16(kc) if kc.shape[0] else None
    dvc = to_dev_bf16(vc) if vc.shape[0] else None
    out = torch.full(dq.shape, float("nan"), dtype=torch.bfloat16, device="cuda")
    P.block_attn(dq, dkc, dvc, dkb, dvb, cache_len, out=out)
    torch.cuda.synchronize()
    got = bits_of(out)
    if kc.shape[0] == 0:
        kc = vc = np.zeros((1, H, 128), np.uint16)
    ref = oracle.block_attn(q, kc, vc, kb, vb, cache_len, rows=rows)
    if rows is not None:
        got = got[rows]
    return attn_errors(got, ref)


def check(errs):
    max_abs, rel_rms = errs
    assert np.isfinite(max_abs) and np.isfinite(rel_rms)
    assert max_abs <= BF16_MAX_ABS, errs
    assert rel_rms <= BF16_REL_RMS, errs


def test_tiny_config_all_rows():
    # 12 heads, 312 query tokens (3 frames of 8x13), cache of 2 blocks (624), 936 keys
    check(run_case(12, 312, 624))


def test_tiny_config_poisoned_padding():
    # cache allocation longer than cache_len, NaN-filled past it: must not be read
    check(run_case(12, 312, 624, cap_extra=100))


@pytest.mark.parametrize("cache_len", [0, 1, 8, 63, 64, 65, 100, 312])
def test_seam_and_tail_positions(cache_len):
    check(run_case(2, 72, cache_len, seed=7 + cache_len, cap_extra=3))


@pytest.mark.parametrize("n_blk,n_q", [(1, 1), (5, 3), (64, 64), (65, 33), (257, 257), (300, 256)])
def test_ragged_sizes(n_blk, n_q):
    check(run_case(3, n_blk, 40, seed=100 + n_blk, n_q=n_q))


def test_jittered_heads_sharp_and_diffuse_softmax():
    check(run_case(12, 312, 624, jitter=True, seed=5))


# ---------------------------------------------------------------- fp32-input check path

def run_case_f32(H, n_blk, cache_len, seed=si.SEED, jitter=False, cap_extra=0, n_q=None):
    import paper_2604_17397_amd as P
    from gpu_util import F32_MAX_ABS
    q, kc, vc, kb, vb = si.attn_inputs(H, n_blk, cache_len, seed=seed, jitter=jitter, dtype="f32",
                                       cache_capacity=cache_len + cap_extra)
    if n_q is not None:
        q = np.ascontiguousarray(q[:n_q])
    dev = lambda a: torch.from_numpy(a).cuda() if a.shape[0] else None
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda")
    P.block_attn(dev(q), dev(kc), dev(vc), dev(kb), dev(vb), cache_len, out=out)
    torch.cuda.synchronize()
    if kc.shape[0] == 0:
        kc = vc = np.zeros((1, H, 128), np.float32)
    ref = oracle.block_attn(q, kc, vc, kb, vb, cache_len)
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref)
    assert np.isfinite(err).all()
    assert err.max() <= F32_MAX_ABS, err.max()


def test_f32_check_tiny_config():
    run_case_f32(12, 312, 624, cap_extra=7)


def test_f32_check_jittered_heads():
    run_case_f32(12, 312, 624, jitter=True, seed=5)


@pytest.mark.parametrize("cache_len,n_blk,n_q", [(0, 72, 72), (1, 5, 3), (31, 33, 33), (32, 64, 1), (100, 129, 129)])
def test_f32_check_seam_and_tails(cache_len, n_blk, n_q):
    run_case_f32(2, n_blk, cache_len, seed=3 + cache_len, cap_extra=2, n_q=n_q)
