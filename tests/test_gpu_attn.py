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


# ---------------------------------------------------------------- lazy running maximum

def structured_case(pattern, n_k_total=700, n_q=70, H=2, amp=40.0, scale=None):
    """Scores with a designed profile along the keys: q = one direction u per row (with a row
    dependent gain), k_j = g(j) * u, so that s_ij ~ gain_i * g(j) * |u|^2 * scale. `pattern`
    picks g: rising (the running maximum must be raised again and again, by far more than the
    kernel's 2^20 overflow limit in total), falling (tile 0 holds the maximum, later
    probabilities underflow), spike_last (one huge logit in the ragged last tile), flat."""
    import paper_2604_17397_amd as P
    rng = np.random.default_rng(11)
    d = 128
    u = rng.standard_normal(d)
    u /= np.linalg.norm(u)
    j = np.arange(n_k_total, dtype=np.float64)
    g = {"rising": amp * j / n_k_total, "falling": amp * (1.0 - j / n_k_total),
         "spike_last": np.where(j == n_k_total - 1, amp, 0.1), "flat": np.full(n_k_total, 0.5)}[pattern]
    gain = np.linspace(0.5, 2.0, n_q) * math_sqrt(d)
    q = np.einsum("i,d->id", gain, u)[:, None, :].repeat(H, axis=1)
    k = np.einsum("j,d->jd", g, u)[:, None, :].repeat(H, axis=1)
    k += 0.01 * rng.standard_normal(k.shape)
    v = rng.standard_normal((n_k_total, H, d))
    c_len = 333
    bits = lambda a: si.f32_to_bf16_bits(a.astype(np.float32))
    qb, kb_all, vb_all = bits(q), bits(k), bits(v)
    kc, kblk, vc, vblk = kb_all[:c_len], kb_all[c_len:], vb_all[:c_len], vb_all[c_len:]
    out = torch.full((n_q, H, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    P.block_attn(to_dev_bf16(qb), to_dev_bf16(kc), to_dev_bf16(vc), to_dev_bf16(kblk), to_dev_bf16(vblk),
                 c_len, out=out, scale=scale)
    torch.cuda.synchronize()
    ref = oracle.block_attn(qb, kc, vc, kblk, vblk, c_len, scale=scale)
    return attn_errors(bits_of(out), ref)


def math_sqrt(x):
    import math
    return math.sqrt(x)


@pytest.mark.parametrize("pattern", ["rising", "falling", "spike_last", "flat"])
@pytest.mark.parametrize("amp", [8.0, 40.0, 150.0])
def test_score_profiles_that_move_the_running_maximum(pattern, amp):
    # amp = 150 gives logits whose exponentials span far more than fp32 can hold relative to
    # tile 0: without a raised maximum the probabilities overflow, with a wrong rescale the
    # output is visibly off.
    check(structured_case(pattern, amp=amp))


def test_softmax_scale_argument():
    check(structured_case("rising", amp=20.0, scale=0.05))
    check(structured_case("flat", scale=0.3))


def test_head_major_strides():
    """q / out / k / v given as [heads, tokens, 128] memory viewed as [tokens, heads, 128]."""
    import paper_2604_17397_amd as P
    H, n_blk, c_len = 3, 150, 200
    q, kc, vc, kb, vb = si.attn_inputs(H, n_blk, c_len, seed=31)
    hm = lambda a: to_dev_bf16(np.ascontiguousarray(a.transpose(1, 0, 2))).transpose(0, 1)
    dq, dkc, dvc, dkb, dvb = hm(q), hm(kc), hm(vc), hm(kb), hm(vb)
    out = torch.full((H, n_blk, 128), float("nan"), dtype=torch.bfloat16, device="cuda").transpose(0, 1)
    assert dq.stride() == (128, n_blk * 128, 1)
    P.block_attn(dq, dkc, dvc, dkb, dvb, c_len, out=out)
    torch.cuda.synchronize()
    ref = oracle.block_attn(q, kc, vc, kb, vb, c_len)
    check(attn_errors(bits_of(out), ref))


def test_random_small_shapes():
    """Thirty seeded draws of (heads, cache_len, n_blk, n_q, jitter, spare cache rows): every row of
    every draw against the oracle. The draws cover several tiles, the seam inside a tile, ragged
    tails, a single key and more query rows than one workgroup holds."""
    rng = np.random.default_rng(20260417)
    for case in range(30):
        H = int(rng.integers(1, 6))
        cache_len = int(rng.choice([0, int(rng.integers(1, 64)), int(rng.integers(64, 400))]))
        n_blk = int(rng.integers(1, 330))
        n_q = int(rng.integers(1, n_blk + 1))
        jitter = bool(rng.integers(0, 2))
        errs = run_case(H, n_blk, cache_len, seed=5000 + case, jitter=jitter, cap_extra=int(rng.integers(0, 5)), n_q=n_q)
        max_abs, rel_rms = errs
        assert np.isfinite(max_abs) and max_abs <= BF16_MAX_ABS and rel_rms <= BF16_REL_RMS, \
            (case, H, cache_len, n_blk, n_q, jitter, errs)
