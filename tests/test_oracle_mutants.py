"""The pins must be able to fail: each plausible mistake, planted in a COPY of the oracle's C
source (one textual edit, compiled to a temporary library, on the CPU), has to be caught by at
least one of the pin tests of tests/test_oracle_attn.py / tests/test_oracle_kv_route.py. The
oracle itself carries no hooks for this."""
import ctypes
import os
import subprocess

import pytest

import oracle
import oracle.oracle as front
from oracle import build as oracle_build

import test_oracle_attn as pins_attn
import test_oracle_kv_route as pins_kv
import test_oracle_rope as pins_rope

SRC = open(oracle_build.SRC).read()

ATTN_PINS = [
    pins_attn.test_weights_sum_to_one_and_are_positive,
    pins_attn.test_single_key_returns_its_value_row,
    pins_attn.test_identical_keys_give_mean_of_values,
    pins_attn.test_two_keys_logistic_closed_form_pins_scale_and_sign,
    pins_attn.test_dominant_key_selects_its_value,
    pins_attn.test_key_value_permutation_invariance,
    lambda: pins_attn.test_seam_invariance(17),
    pins_attn.test_key_shift_invariance,
    lambda: pins_attn.test_brute_force_tiny(4),
    lambda: pins_attn.test_library_sdpa_float64("bf16"),
]
KV_PINS = [
    pins_kv.test_commit_sequence_equals_concatenation,
    pins_kv.test_commit_writes_only_its_slot,
    pins_kv.test_commit_is_append_only_and_bounded,
    pins_kv.test_rollback_restores_prefix_and_scrubs,
    pins_kv.test_rollback_then_commit_leaves_no_trace,
]
ROUTE_PINS = [
    pins_kv.test_route_is_min_threshold_and_force_reject,
    pins_kv.test_route_tie_accepts,
    pins_kv.test_route_min_equals_all_frames_pass_bruteforce,
    pins_kv.test_route_min_catches_one_bad_frame_that_mean_masks,
    pins_kv.test_route_nan_and_signed_zero,
    pins_kv.test_mean_route_exact_values_and_closed_form_accept_probability,
    pins_kv.test_mean_route_of_opposite_infinities_is_the_canonical_nan,
]

ROPE_PINS = [
    pins_rope.test_zero_angle_is_the_identity_and_quarter_turn_swaps_the_pair,
    pins_rope.test_matches_complex_multiplication_in_float64,
    pins_rope.test_norm_is_preserved_and_rotations_compose,
    pins_rope.test_relative_position_property,
    pins_rope.test_worked_example_by_hand,
]

# (name, text to find (must occur exactly `count` times), replacement, which occurrence, pins)
MUTANTS = [
    ("dropped softmax scale", "s[j] = dot * scale;", "s[j] = dot;", 1, 0, ATTN_PINS),
    ("negated logits", "s[j] = exp(s[j] - m);", "s[j] = exp(m - s[j]);", 1, 0, ATTN_PINS),
    ("missing normalisation", "for (int64_t t = 0; t < head_dim; ++t) o[t] /= z;", ";", 1, 0, ATTN_PINS),
    ("query dims reversed", "widen(q, qoff + t, dtype)", "widen(q, qoff + (head_dim - 1 - t), dtype)", 1, 0,
     ATTN_PINS),
    ("block keys in reverse order (values not)", ": (j - cache_len) * blk_token_stride + h * blk_head_stride;",
     ": (n_k - 1 - j) * blk_token_stride + h * blk_head_stride;", 2, 0, ATTN_PINS),
    ("last key left out of the sums", "for (int64_t j = 0; j < n_k; ++j) {\n          s[j] = exp(s[j] - m);",
     "s[n_k - 1] = 0.0;\n        for (int64_t j = 0; j < n_k - 1; ++j) {\n          s[j] = exp(s[j] - m);", 1, 0,
     ATTN_PINS),
    ("values of the block taken from the cache side stride", "const void *vb = (j < cache_len) ? v_cache : v_blk;",
     "const void *vb = (j < cache_len) ? v_cache : k_blk;", 1, 0, ATTN_PINS),
    ("commit writes the slot after the one asked for",
     "((l * capacity_tokens + slot * block_tokens + t) * n_heads + h) * head_dim + x;",
     "((l * capacity_tokens + slot * block_tokens + (t + 1) % block_tokens) * n_heads + h) * head_dim + x;", 1, 0,
     KV_PINS),
    ("commit forgets V", "cache_v[dst] = v_blk[src];", "cache_v[dst] = k_blk[src];", 1, 0, KV_PINS),
    ("rollback keeps the old length", "*cache_len = new_len;", ";", 1, 0, KV_PINS),
    ("rollback does not scrub", "cache_k[dst] = 0;", ";", 1, 0, KV_PINS),
    ("strict threshold", "qb >= tau", "qb > tau", 1, 0, ROUTE_PINS),
    ("block 0 not force-rejected", "(block_idx != 0 && qb >= tau)", "(qb >= tau)", 1, 0, ROUTE_PINS),
    ("max instead of min", "if (s < qb || (s == qb && signbit(s) && !signbit(qb))) qb = s;",
     "if (s > qb) qb = s;", 1, 0, ROUTE_PINS),
    ("mean summed in fp32", "acc += (double)scores[i];", "acc = (double)((float)acc + scores[i]);", 1, 0,
     ROUTE_PINS),
    ("mean of +inf and -inf leaves a raw NaN", "if (isnan(qb)) {", "if (0) {", 1, 0, ROUTE_PINS),
    ("rotation the other way round", "out[e] = bf16_rne(fmaf(re, c, -im_sin));", "out[e] = bf16_rne(fmaf(re, c, im_sin));", 1, 0,
     ROPE_PINS),
    ("imaginary part forgets the cosine term", "out[e + 1] = bf16_rne(fmaf(re, sn, im_cos));",
     "out[e + 1] = bf16_rne(re * sn);", 1, 0, ROPE_PINS),
    ("pairs taken as first half / second half", "const int64_t e = (t * n_heads + h) * head_dim + 2 * i;\n        const float re = (float)widen(x, e, ORACLE_BF16), im = (float)widen(x, e + 1, ORACLE_BF16);",
     "const int64_t e = (t * n_heads + h) * head_dim + 2 * i;\n        const float re = (float)widen(x, (t * n_heads + h) * head_dim + i, ORACLE_BF16), im = (float)widen(x, (t * n_heads + h) * head_dim + half + i, ORACLE_BF16);",
     1, 0, ROPE_PINS),
    ("angle table indexed by head instead of token", "const float c = cos_t[t * half + i], sn = sin_t[t * half + i];",
     "const float c = cos_t[(h % n_tokens) * half + i], sn = sin_t[(h % n_tokens) * half + i];", 1, 0, ROPE_PINS),
    ("bf16 rounding truncates", "u += 0x7FFFu + ((u >> 16) & 1u);", ";", 1, 0, ROPE_PINS),
]


@pytest.mark.parametrize("name,find,repl,count,which,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, name, find, repl, count, which, pins):
    assert SRC.count(find) == count, "the oracle source changed: update this mutant's pattern"
    pos = -1
    for _ in range(which + 1):
        pos = SRC.index(find, pos + 1)
    mutated = SRC[:pos] + repl + SRC[pos + len(find):]
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(mutated)
    subprocess.run(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(lib), str(src), "-lm"],
                   check=True)
    # the front-end loads whatever build() names; point it at the mutant for this test only
    monkeypatch.setattr(front, "_LIB", None)
    monkeypatch.setattr(front._build, "build", lambda force=False: str(lib))
    caught = []
    for pin in pins:
        try:
            pin()
        except AssertionError:
            caught.append(pin)
    monkeypatch.setattr(front, "_LIB", None)   # the next test reloads the real oracle
    assert caught, "no pin noticed the planted mistake: " + name
