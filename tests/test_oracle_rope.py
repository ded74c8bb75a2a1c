"""Pins of the oracle's rotary embedding (paper Sec. 4.1 "Models" names RoPE only; the reading --
rotation of consecutive pairs by caller-supplied angles, fp32 arithmetic in a fixed order, bf16
result -- is stated at oracle/sdvg_oracle.c). Closed forms, the defining relative-position
property, norm preservation, composition, and complex multiplication in fp64 by numpy."""
import math

import numpy as np

import oracle
import sdvg_inputs as si

f64 = si.bf16_bits_to_f64


def bf(a):
    return si.f32_to_bf16_bits(np.asarray(a, np.float32))


def tables(angles):
    return np.cos(angles).astype(np.float32), np.sin(angles).astype(np.float32)


def test_zero_angle_is_the_identity_and_quarter_turn_swaps_the_pair():
    x = si.normal_bf16(700, 0, (9, 3, 128))
    one, zero = np.ones((9, 64), np.float32), np.zeros((9, 64), np.float32)
    assert np.array_equal(oracle.rope(x, one, zero), x)
    y = f64(oracle.rope(x, zero, one))               # angle pi/2: (re, im) -> (-im, re), exactly
    xx = f64(x)
    assert np.array_equal(y[..., 0::2], -xx[..., 1::2]) and np.array_equal(y[..., 1::2], xx[..., 0::2])
    y = f64(oracle.rope(x, -one, zero))              # angle pi: negation
    assert np.array_equal(y, -xx)


def test_matches_complex_multiplication_in_float64():
    rng = np.random.default_rng(5)
    n, H, d = 37, 4, 128
    x = si.normal_bf16(701, 0, (n, H, d))
    ang = rng.uniform(-50, 50, (n, d // 2))
    c, s = tables(ang)
    got = f64(oracle.rope(x, c, s))
    xx = f64(x)
    z = (xx[..., 0::2] + 1j * xx[..., 1::2]) * (c.astype(np.float64) + 1j * s.astype(np.float64))[:, None, :]
    want = np.empty_like(xx)
    want[..., 0::2], want[..., 1::2] = z.real, z.imag
    # fp32 arithmetic then bf16 rounding: within one bf16 ulp of the exact product of the same tables
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 2.0 ** -8 * np.abs(xx).max() * 2.0 ** -7)
    # and the pair convention is "consecutive elements", not "first half / second half"
    half = np.empty_like(xx)
    zh = (xx[..., :d // 2] + 1j * xx[..., d // 2:]) * (c.astype(np.float64) + 1j * s.astype(np.float64))[:, None, :]
    half[..., :d // 2], half[..., d // 2:] = zh.real, zh.imag
    assert np.abs(got - half).max() > 0.5


def test_norm_is_preserved_and_rotations_compose():
    n, H, d = 21, 2, 128
    x = si.normal_bf16(702, 0, (n, H, d))
    rng = np.random.default_rng(6)
    a, b = rng.uniform(-3, 3, (n, d // 2)), rng.uniform(-3, 3, (n, d // 2))
    xa = oracle.rope(x, *tables(a))
    pair_norm = lambda v: np.hypot(f64(v)[..., 0::2], f64(v)[..., 1::2])
    assert np.allclose(pair_norm(xa), pair_norm(x), rtol=2.0 ** -7, atol=1e-3)
    xab = f64(oracle.rope(xa, *tables(b)))
    direct = f64(oracle.rope(x, *tables(a + b)))
    assert np.abs(xab - direct).max() <= 2.0 ** -6 * np.abs(direct).max()


def test_relative_position_property():
    # The point of RoPE: <rope(q, p1), rope(k, p2)> depends on p1 - p2 only. Angles p * theta_i.
    d, H = 128, 1
    theta = 10000.0 ** (-np.arange(d // 2) / (d // 2))
    q = si.normal_bf16(703, 0, (1, H, d))
    k = si.normal_bf16(703, 1, (1, H, d))

    def dot(p1, p2):
        rq = f64(oracle.rope(q, *tables((p1 * theta)[None])))
        rk = f64(oracle.rope(k, *tables((p2 * theta)[None])))
        return float((rq * rk).sum())
    base = dot(7.0, 3.0)
    scale = float(np.abs(f64(q)).max() * np.abs(f64(k)).max() * d)
    for shift in (1.0, 10.0, 100.0, 1000.0):
        assert abs(dot(7.0 + shift, 3.0 + shift) - base) <= 2.0 ** -7 * scale * 0.2
    assert abs(dot(8.0, 3.0) - base) > 1e-3 * scale * 0.01     # a different offset does change it


def test_worked_example_by_hand():
    # one pair, 3-4-5 rotation: (re, im) = (1, 2), cos = 0.6, sin = 0.8 (as fp32) ->
    # re' = 0.6 - 1.6 = -1.0, im' = 0.8 + 1.2 = 2.0 up to fp32 rounding of the tables, then bf16
    x = bf(np.array([[[1.0, 2.0]]]))
    y = f64(oracle.rope(x, np.array([[0.6]], np.float32), np.array([[0.8]], np.float32)))
    assert y.shape == (1, 1, 2) and abs(y[0, 0, 0] + 1.0) <= 2.0 ** -8 and abs(y[0, 0, 1] - 2.0) <= 2.0 ** -7
    # rounding to bf16 is to nearest even: 1 + 2^-8 (a tie) goes to 1, 1 + 3 * 2^-8 (a tie) to 1 + 2^-6
    x = bf(np.array([[[1.0, 0.0]]]))
    for cosv, want in ((1.0 + 2.0 ** -8, 1.0), (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6), (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7)):
        y = f64(oracle.rope(x, np.array([[cosv]], np.float32), np.array([[0.0]], np.float32)))
        assert y[0, 0, 0] == want, (cosv, y[0, 0, 0])
