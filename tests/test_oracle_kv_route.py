"""Pins for the KV commit / rollback mirror and the worst-frame router oracle."""
import math

import numpy as np
import pytest

import oracle
import sdvg_inputs as si

L, H, D, T, CAP = 3, 2, 8, 5, 20


def blk(seed):
    rng = np.random.default_rng(seed)
    return (rng.integers(1, 65535, size=(L, T, H, D), dtype=np.uint16),
            rng.integers(1, 65535, size=(L, T, H, D), dtype=np.uint16))


def test_commit_sequence_equals_concatenation():
    m = oracle.KVMirror(L, CAP, H, D, T, fill=0xABCD)
    blocks = [blk(s) for s in range(4)]
    for s, (k, v) in enumerate(blocks):
        assert oracle.kv_commit(m, k, v, s) == 0
        assert m.cache_len == (s + 1) * T
    assert np.array_equal(m.k[:, :4 * T], np.concatenate([b[0] for b in blocks], axis=1))
    assert np.array_equal(m.v[:, :4 * T], np.concatenate([b[1] for b in blocks], axis=1))
    # nothing outside the committed slots was touched (canary fill)
    assert np.all(m.k[:, 4 * T:] == 0xABCD) and np.all(m.v[:, 4 * T:] == 0xABCD)


def test_commit_writes_only_its_slot():
    m = oracle.KVMirror(L, CAP, H, D, T, fill=0x1111)
    k0, v0 = blk(0)
    oracle.kv_commit(m, k0, v0, 0)
    before_k, before_v = m.k.copy(), m.v.copy()
    k1, v1 = blk(1)
    oracle.kv_commit(m, k1, v1, 1)
    changed = (m.k != before_k) | (m.v != before_v)
    assert not changed[:, :T].any() and not changed[:, 2 * T:].any()
    assert np.array_equal(m.k[:, T:2 * T], k1) and np.array_equal(m.v[:, T:2 * T], v1)
    # k and v are not swapped
    assert not np.array_equal(m.k[:, T:2 * T], v1)


def test_commit_is_append_only_and_bounded():
    m = oracle.KVMirror(L, CAP, H, D, T)
    k, v = blk(0)
    assert oracle.kv_commit(m, k, v, 1) == -3      # slot 0 not yet filled
    assert oracle.kv_commit(m, k, v, -1) == -3
    assert m.cache_len == 0 and not m.k.any()
    for s in range(CAP // T):
        assert oracle.kv_commit(m, k, v, s) == 0
    assert oracle.kv_commit(m, k, v, CAP // T) == -3  # full
    assert m.cache_len == CAP


def test_rollback_restores_prefix_and_scrubs():
    m = oracle.KVMirror(L, CAP, H, D, T)
    for s in range(2):
        oracle.kv_commit(m, *blk(s), s)
    snap_k, snap_v = m.k.copy(), m.v.copy()
    oracle.kv_commit(m, *blk(7), 2)
    assert oracle.kv_rollback(m, 2 * T) == 0
    assert m.cache_len == 2 * T
    assert np.array_equal(m.k, snap_k) and np.array_equal(m.v, snap_v)   # scrubbed range is zero again
    # rollback to current length is a no-op; growing or negative is an error
    assert oracle.kv_rollback(m, 2 * T) == 0 and np.array_equal(m.k, snap_k)
    assert oracle.kv_rollback(m, 2 * T + 1) == -3
    assert oracle.kv_rollback(m, -1) == -3
    # partial-block rollback zeroes exactly [new_len, old_len)
    assert oracle.kv_rollback(m, T + 2) == 0
    assert np.array_equal(m.k[:, :T + 2], snap_k[:, :T + 2]) and not m.k[:, T + 2:].any()
    # re-commit of different data leaves no trace of the old block... slot index must match length
    assert oracle.kv_commit(m, *blk(9), 1) == -3


def test_rollback_then_commit_leaves_no_trace():
    m = oracle.KVMirror(L, CAP, H, D, T)
    oracle.kv_commit(m, *blk(0), 0)
    oracle.kv_commit(m, *blk(1), 1)
    oracle.kv_rollback(m, T)
    k2, v2 = blk(2)
    oracle.kv_commit(m, k2, v2, 1)
    m2 = oracle.KVMirror(L, CAP, H, D, T)
    oracle.kv_commit(m2, *blk(0), 0)
    oracle.kv_commit(m2, k2, v2, 1)
    assert np.array_equal(m.k, m2.k) and np.array_equal(m.v, m2.v)


# ---------------------------------------------------------------- routing (Sec. 3 Eq. 1)

def test_route_is_min_threshold_and_force_reject():
    s = np.array([0.3, -0.2, 1.5, -0.69, 0.0], np.float32)
    dec, qb = oracle.route(s, -0.7, 3)
    assert dec == 1 and qb == np.float32(-0.69)
    dec, qb = oracle.route(s, -0.6, 3)
    assert dec == 0 and qb == np.float32(-0.69)
    # block 0 is rejected whatever the scores, but q_b is still the true minimum
    dec, qb = oracle.route(s, -0.7, 0)
    assert dec == 0 and qb == np.float32(-0.69)
    dec, qb = oracle.route(np.full(12, np.inf, np.float32), -0.7, 0)
    assert dec == 0 and qb == np.inf


def test_route_tie_accepts():
    tau = np.float32(-0.7)
    dec, qb = oracle.route(np.array([0.1, tau, 0.5], np.float32), float(tau), 1)
    assert dec == 1 and qb == tau
    below = np.nextafter(tau, np.float32(-np.inf), dtype=np.float32)
    dec, _ = oracle.route(np.array([0.1, below, 0.5], np.float32), float(tau), 1)
    assert dec == 0


def test_route_min_equals_all_frames_pass_bruteforce():
    rng = np.random.default_rng(3)
    for _ in range(2000):
        F = int(rng.integers(1, 20))
        s = rng.normal(-0.3, 0.6, F).astype(np.float32)
        tau = float(np.float32(rng.normal(-0.7, 0.5)))
        b = int(rng.integers(0, 3))
        dec, qb = oracle.route(s, tau, b)
        assert qb == s.min()
        assert dec == int(b != 0 and all(x >= np.float32(tau) for x in s))
        # permutation invariance
        dec2, qb2 = oracle.route(rng.permutation(s), tau, b)
        assert (dec2, qb2) == (dec, qb)


def test_route_monotone_in_tau():
    # Table 1: the accept rate rises as tau falls; per block the decision is monotone in tau.
    scores = si.frame_scores_correlated(5, 500)
    taus = [-2.5, -2.0, -1.5, -1.0, -0.9, -0.8, -0.7]
    prev = None
    for tau in taus:
        dec = np.array([oracle.route(scores[i], tau, 1)[0] for i in range(500)])
        if prev is not None:
            assert np.all(dec <= prev)
        prev = dec
    assert prev.sum() < 500 and prev.sum() > 0


def test_route_min_catches_one_bad_frame_that_mean_masks():
    # Sec. 3 "Worst-frame aggregation" / Sec. 4.3: one degraded frame rejects under min.
    s = np.array([0.5] * 11 + [-3.0], np.float32)
    assert oracle.route(s, -0.7, 2)[0] == 0
    dec, qb = oracle.route(s, -0.7, 2, mode="mean")
    assert dec == 1 and abs(float(qb) - (0.5 * 11 - 3.0) / 12) < 1e-7


def test_route_nan_and_signed_zero():
    dec, qb = oracle.route(np.array([0.2, np.nan, 0.1], np.float32), -10.0, 1)
    assert dec == 0 and qb.view(np.uint32) == 0x7FC00000
    for order in ([0.0, -0.0, 1.0], [-0.0, 0.0, 1.0], [1.0, 0.0, -0.0]):
        dec, qb = oracle.route(np.array(order, np.float32), 0.0, 1)
        assert dec == 1 and qb.view(np.uint32) == 0x80000000   # -0.0 is the minimum; -0.0 >= 0.0
    dec, qb = oracle.route(np.array([-np.inf, 1.0], np.float32), -1e30, 1)
    assert dec == 0 and qb == -np.inf


def test_iid_score_generator_matches_closed_form_accept_probability():
    # P(accept) = (1 - Phi((tau - mean)/std))^F for i.i.d. N(mean, std) frames: pins the
    # generator and the router together (4-sigma binomial band).
    n = 200_000
    scores = si.frame_scores_iid(42, n)
    qmin = scores.min(axis=1)
    for tau in (-1.0, -0.7):
        p = (1 - 0.5 * (1 + math.erf((tau + 0.3) / 0.6 / math.sqrt(2)))) ** 12
        acc = sum(oracle.route(scores[i], tau, 1)[0] for i in range(0, n, 10)) / (n // 10)
        band = 4 * math.sqrt(p * (1 - p) / (n // 10))
        assert abs(acc - p) < band
        assert abs((qmin >= np.float32(tau)).mean() - p) < 4 * math.sqrt(p * (1 - p) / n)


def test_table1_ordering_property_holds_for_router():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "table1_tau_accept.txt")
    rows = [tuple(map(float, ln.split())) for ln in open(path) if ln.strip() and ln[0] != "#"]
    taus = [r[0] for r in rows]
    paper_rates = [r[1] for r in rows]
    assert taus == sorted(taus, reverse=True) and paper_rates == sorted(paper_rates)
    scores = si.frame_scores_correlated(7, 2000)
    ours = [np.mean([oracle.route(scores[i], t, 1 + i % 8)[0] for i in range(2000)]) for t in taus]
    assert ours == sorted(ours) and ours[-1] > ours[0]


def test_mean_route_exact_values_and_closed_form_accept_probability():
    # Sec. 4.3 "Min-frame vs. average-frame scoring": the ablation's router. Exact pins: means
    # that are representable (or whose correctly rounded fp32 value is known), the accept rule
    # and block 0; statistical pin: the mean of F i.i.d. N(mu, sigma) rewards is N(mu, sigma/sqrt(F)),
    # so P(accept) = 1 - Phi((tau - mu) sqrt(F) / sigma).
    dec, qb = oracle.route(np.array([1.0, 2.0, 3.0, 6.0], np.float32), 3.0, 1, mode="mean")
    assert dec == 1 and qb == np.float32(3.0)
    dec, qb = oracle.route(np.array([1.0, 2.0, 3.0, 6.0], np.float32), 3.0, 0, mode="mean")
    assert dec == 0 and qb == np.float32(3.0)
    dec, qb = oracle.route(np.array([0.5, 0.25, 0.25], np.float32), 0.3334, 2, mode="mean")
    assert dec == 0 and qb.view(np.uint32) == np.float32(1.0 / 3.0).view(np.uint32)
    # a sum that fp32 accumulation would get wrong: 2^24 + 1 + 1 - 2^24 = 2 exactly in fp64
    dec, qb = oracle.route(np.array([16777216.0, 1.0, 1.0, -16777216.0], np.float32), 0.5, 1, mode="mean")
    assert dec == 1 and qb == np.float32(0.5)
    dec, qb = oracle.route(np.array([0.2, np.nan, 0.1], np.float32), -10.0, 1, mode="mean")
    assert dec == 0 and qb.view(np.uint32) == 0x7FC00000
    n = 60_000
    scores = si.frame_scores_iid(43, n)
    for tau in (-0.5, -0.3, -0.2):
        p = 1 - 0.5 * (1 + math.erf((tau + 0.3) * math.sqrt(12) / 0.6 / math.sqrt(2)))
        acc = sum(oracle.route(scores[i], tau, 1, mode="mean")[0] for i in range(0, n, 3)) / (n // 3)
        assert abs(acc - p) < 4 * math.sqrt(p * (1 - p) / (n // 3)) + 1e-3


def test_mean_route_of_opposite_infinities_is_the_canonical_nan():
    # +inf and -inf among the rewards: the fp64 sum is NaN. Reading taken (the paper is silent):
    # such a block is unscorable, so it rejects and reports the canonical quiet NaN, exactly as a
    # NaN reward does. One infinity alone stays an ordinary value.
    for s in ([np.inf, -np.inf], [0.5, -np.inf, np.inf, 1.0], [np.inf, 2.0, -np.inf]):
        dec, qb = oracle.route(np.array(s, np.float32), -1e30, 3, mode="mean")
        assert dec == 0 and qb.view(np.uint32) == 0x7FC00000
    dec, qb = oracle.route(np.array([np.inf, 1.0], np.float32), 0.0, 3, mode="mean")
    assert dec == 1 and qb == np.inf
    dec, qb = oracle.route(np.array([-np.inf, 1.0], np.float32), 0.0, 3, mode="mean")
    assert dec == 0 and qb == -np.inf
    # the minimum of the same scores is an ordinary -inf, not a NaN
    dec, qb = oracle.route(np.array([np.inf, -np.inf], np.float32), 0.0, 3)
    assert dec == 0 and qb == -np.inf


def test_buffer_copy_is_a_byte_copy_and_touches_nothing_else():
    # Sec. 3 "Inference flow": clone before scoring, restore on rejection. Pins: the copy equals
    # numpy's own slice assignment, leaves the bytes around it alone, and clone -> mutate ->
    # restore returns the original bytes.
    rng = np.random.default_rng(5)
    for n in (0, 1, 15, 16, 17, 4099):
        src = rng.integers(0, 256, n + 7, dtype=np.uint8)
        dst = np.full(n + 9, 0xA5, np.uint8)
        want = dst.copy()
        want[:n] = src[:n]
        assert oracle.buffer_copy(dst, src, n) == 0
        assert np.array_equal(dst, want)
    live = rng.integers(0, 256, 1000, dtype=np.uint8)
    orig = live.copy()
    snap = np.zeros_like(live)
    oracle.buffer_copy(snap, live)
    live[::3] ^= 0xFF
    oracle.buffer_copy(live, snap)
    assert np.array_equal(live, orig)
