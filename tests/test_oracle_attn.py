"""Pins for the attention oracle: closed forms, invariants, a library routine and brute force.

Each test is chosen so that a plausible mistake in oracle/sdvg_oracle.c (wrong scale, wrong
sign, transposed operand, dropped term, cache/block seam off by one, wrong stride) fails it.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import sdvg_inputs as si

D = 128


def bf(x):
    return si.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def rand_case(seed, n_q, c, n_blk, H=3, d=D, scale_q=1.0):
    q = si.normal_bf16(seed, 0, (n_q, H, d)) if scale_q == 1.0 else bf(
        scale_q * si.normal_f32(seed, 0, (n_q, H, d)))
    kc = si.normal_bf16(seed, 1, (max(c, 1), H, d))
    vc = si.normal_bf16(seed, 2, (max(c, 1), H, d))
    kb = si.normal_bf16(seed, 3, (n_blk, H, d))
    vb = si.normal_bf16(seed, 4, (n_blk, H, d))
    return q, kc, vc, kb, vb


def test_weights_sum_to_one_and_are_positive():
    q, kc, vc, kb, vb = rand_case(1, 5, 9, 7)
    out, w = oracle.block_attn(q, kc, vc, kb, vb, 9, return_weights=True)
    assert w.shape == (5, 3, 16)
    assert np.all(w >= 0)
    assert np.max(np.abs(w.sum(-1) - 1.0)) < 1e-14
    # and out really is the weighted sum of [cache; block] values
    V = np.concatenate([si.bf16_bits_to_f64(vc[:9]), si.bf16_bits_to_f64(vb)], 0)
    ref = np.einsum("qhk,khd->qhd", w, V)
    assert np.max(np.abs(out - ref)) < 1e-13


def test_single_key_returns_its_value_row():
    q, kc, vc, kb, vb = rand_case(2, 4, 0, 1)
    out = oracle.block_attn(q, kc, vc, kb, vb, 0)
    v = si.bf16_bits_to_f64(vb)[0]
    assert np.array_equal(out, np.broadcast_to(v, out.shape))
    # single key living in the cache side
    q, kc, vc, kb, vb = rand_case(3, 4, 1, 1)
    kb2 = kb.copy(); vb2 = vb.copy()
    # make the block key hugely unfavourable instead of absent is a different test; here use
    # cache_len=1 with a block key identical to the cache key and value -> still that value
    kb2[0] = kc[0]; vb2[0] = vc[0]
    out = oracle.block_attn(q, kc, vc, kb2, vb2, 1)
    v = si.bf16_bits_to_f64(vc)[0]
    assert np.max(np.abs(out - v)) < 1e-15


def test_identical_keys_give_mean_of_values():
    H, n_k = 2, 11
    q = si.normal_bf16(4, 0, (3, H, D))
    key = si.normal_bf16(4, 1, (1, H, D))
    kc = np.repeat(key, 6, axis=0); kb = np.repeat(key, 5, axis=0)
    vc = si.normal_bf16(4, 2, (6, H, D)); vb = si.normal_bf16(4, 4, (5, H, D))
    out = oracle.block_attn(q, kc, vc, kb, vb, 6)
    mean = np.concatenate([si.bf16_bits_to_f64(vc), si.bf16_bits_to_f64(vb)], 0).mean(0)
    assert np.max(np.abs(out - mean)) < 1e-14


def test_zero_query_gives_mean_of_values():
    q, kc, vc, kb, vb = rand_case(5, 2, 8, 4)
    q[:] = 0
    out = oracle.block_attn(q, kc, vc, kb, vb, 8)
    mean = np.concatenate([si.bf16_bits_to_f64(vc[:8]), si.bf16_bits_to_f64(vb)], 0).mean(0)
    assert np.max(np.abs(out - mean)) < 1e-14


def test_equal_values_pass_through():
    q, kc, vc, kb, vb = rand_case(6, 3, 5, 6)
    row = si.normal_bf16(6, 9, (1, 3, D))
    vc[:] = row; vb[:] = row
    out = oracle.block_attn(q, kc, vc, kb, vb, 5)
    assert np.max(np.abs(out - si.bf16_bits_to_f64(row))) < 1e-14


def test_two_keys_logistic_closed_form_pins_scale_and_sign():
    # With two keys the weight of key 0 is the logistic function of the logit gap.
    # q = a*e0, k0 = b*e0, k1 = -b*e0  ->  gap = 2ab/sqrt(d); values are +-1 vectors.
    H = 1
    a, b = 3.0, 2.0
    q = np.zeros((1, H, D), np.float32); q[0, 0, 0] = a
    k = np.zeros((2, H, D), np.float32); k[0, 0, 0] = b; k[1, 0, 0] = -b
    v = np.zeros((2, H, D), np.float32); v[0] = 1.0; v[1] = -1.0
    gap = 2 * a * b / math.sqrt(D)
    w0 = 1.0 / (1.0 + math.exp(-gap))
    expect = w0 * 1.0 + (1 - w0) * -1.0   # = tanh(gap/2)
    assert abs(expect - math.tanh(gap / 2)) < 1e-15
    # key 0 in the cache, key 1 in the block
    out = oracle.block_attn(bf(q), bf(k[:1]), bf(v[:1]), bf(k[1:]), bf(v[1:]), 1)
    assert np.max(np.abs(out - expect)) < 1e-15
    # both in the block, order swapped -> sign flips
    out = oracle.block_attn(bf(q), bf(k[:1]), bf(v[:1]), bf(k[::-1].copy()), bf(v[::-1].copy()), 0)
    assert np.max(np.abs(out - expect)) < 1e-15
    # explicit scale argument is honoured
    out = oracle.block_attn(bf(q), bf(k[:1]), bf(v[:1]), bf(k[1:]), bf(v[1:]), 1, scale=0.5)
    assert np.max(np.abs(out - math.tanh(0.5 * 2 * a * b / 2))) < 1e-15


def test_dominant_key_selects_its_value():
    q, kc, vc, kb, vb = rand_case(7, 2, 6, 6, H=2)
    # make block key 3 equal to 8*q for row 0 / head 0: logit ~ 8*|q|^2/sqrt(d) ~ 90
    qf = si.bf16_bits_to_f64(q)
    kb[3, 0] = bf(8.0 * qf[0, 0])
    out = oracle.block_attn(q, kc, vc, kb, vb, 6, rows=[0])
    assert np.max(np.abs(out[0, 0] - si.bf16_bits_to_f64(vb)[3, 0])) < 1e-12


def test_key_value_permutation_invariance():
    q, kc, vc, kb, vb = rand_case(8, 4, 10, 6)
    out = oracle.block_attn(q, kc, vc, kb, vb, 10)
    K = np.concatenate([kc[:10], kb], 0); V = np.concatenate([vc[:10], vb], 0)
    perm = np.random.default_rng(0).permutation(16)
    K2, V2 = K[perm], V[perm]
    out2 = oracle.block_attn(q, K2[:10].copy(), V2[:10].copy(), K2[10:].copy(), V2[10:].copy(), 10)
    assert np.max(np.abs(out - out2)) < 1e-13
    # permuting keys WITHOUT values must change the result (the test has teeth)
    out3 = oracle.block_attn(q, K2[:10].copy(), V[:10].copy(), K2[10:].copy(), V[10:].copy(), 10)
    assert np.max(np.abs(out - out3)) > 1e-3


@pytest.mark.parametrize("c", [0, 1, 15, 16, 17, 20, 39])
def test_seam_invariance(c):
    # For fixed total K, V every split point between "cache" and "block" gives the same out.
    n_k, H = 40, 2
    q = si.normal_bf16(9, 0, (3, H, D))
    K = si.normal_bf16(9, 1, (n_k, H, D)); V = si.normal_bf16(9, 2, (n_k, H, D))
    base = oracle.block_attn(q, K[:1], V[:1], K, V, 0)
    kc = K[:max(c, 1)].copy(); vc = V[:max(c, 1)].copy()
    out = oracle.block_attn(q, kc, vc, K[c:].copy(), V[c:].copy(), c)
    assert np.max(np.abs(out - base)) < 1e-13


def test_key_shift_invariance():
    # adding u to every key shifts all logits of a row equally -> output unchanged
    H = 2
    q = si.normal_f32(10, 0, (3, H, D))
    K = si.normal_f32(10, 1, (12, H, D)); V = si.normal_f32(10, 2, (12, H, D))
    u = si.normal_f32(10, 7, (1, H, D))
    a = oracle.block_attn(q, K[:5].copy(), V[:5].copy(), K[5:].copy(), V[5:].copy(), 5)
    K2 = (K.astype(np.float64) + u).astype(np.float32)  # fp32 path so the shift is representable
    b = oracle.block_attn(q, K2[:5].copy(), V[:5].copy(), K2[5:].copy(), V[5:].copy(), 5)
    assert np.max(np.abs(a - b)) < 1e-5   # fp32 rounding of K+u, not of the oracle


def test_cache_tokens_past_cache_len_are_ignored():
    q, kc, vc, kb, vb = si.attn_inputs(2, 5, 7, cache_capacity=12, seed=11)
    assert np.isnan(si.bf16_bits_to_f64(kc[7:])).all()
    out = oracle.block_attn(q, kc, vc, kb, vb, 7)
    assert np.isfinite(out).all()
    out2 = oracle.block_attn(q, kc[:7].copy(), vc[:7].copy(), kb, vb, 7)
    assert np.array_equal(out, out2)


def test_strided_views_match_dense():
    # head-major storage seen through token-major logical views
    q, kc, vc, kb, vb = rand_case(12, 4, 6, 5)
    dense = oracle.block_attn(q, kc, vc, kb, vb, 6)
    hm = lambda a: np.ascontiguousarray(a.transpose(1, 0, 2)).transpose(1, 0, 2)
    out = oracle.block_attn(hm(q), hm(kc), hm(vc), hm(kb), hm(vb), 6)
    assert not hm(q).flags.c_contiguous
    assert np.array_equal(out, dense)


def test_row_subset_matches_full():
    q, kc, vc, kb, vb = rand_case(13, 9, 6, 9)
    full = oracle.block_attn(q, kc, vc, kb, vb, 6)
    sub = oracle.block_attn(q, kc, vc, kb, vb, 6, rows=[8, 0, 3])
    assert np.array_equal(sub, full[[8, 0, 3]])


def brute(q, K, V, scale):
    """Explicit P matrix with python loops (tiny shapes only)."""
    n_q, H, d = q.shape
    out = np.zeros((n_q, H, d))
    for h in range(H):
        for i in range(n_q):
            logits = [scale * sum(q[i, h, t] * K[j, h, t] for t in range(d)) for j in range(K.shape[0])]
            m = max(logits)
            e = [math.exp(x - m) for x in logits]
            z = sum(e)
            for t in range(d):
                out[i, h, t] = sum(e[j] * V[j, h, t] for j in range(K.shape[0])) / z
    return out


@pytest.mark.parametrize("d", [4, 128])
def test_brute_force_tiny(d):
    n_q, c, n_blk, H = 3, 3, 5, 2
    q, kc, vc, kb, vb = rand_case(14, n_q, c, n_blk, H=H, d=d)
    out = oracle.block_attn(q, kc, vc, kb, vb, c)
    f = si.bf16_bits_to_f64
    ref = brute(f(q), np.concatenate([f(kc[:c]), f(kb)]), np.concatenate([f(vc[:c]), f(vb)]),
                1.0 / math.sqrt(d))
    assert np.max(np.abs(out - ref)) < 1e-13


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_library_sdpa_float64(dtype):
    # Library special case: torch's scaled_dot_product_attention on CPU in float64.
    H, n_q, c = 4, 37, 50
    q, kc, vc, kb, vb = si.attn_inputs(H, n_q, c, seed=15, dtype=dtype, jitter=True)
    out = oracle.block_attn(q, kc, vc, kb, vb, c)
    f = si.bf16_bits_to_f64 if dtype == "bf16" else (lambda a: a.astype(np.float64))
    tq = torch.from_numpy(f(q)).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.concatenate([f(kc), f(kb)])).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.concatenate([f(vc), f(vb)])).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].permute(1, 0, 2).numpy()
    assert ref.dtype == np.float64
    assert np.max(np.abs(out - ref)) < 1e-12
