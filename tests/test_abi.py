"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments on the host before touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import paper_2604_17397_amd as pkg
    if not os.path.exists(pkg.binding.LIB_PATH):
        from paper_2604_17397_amd import build
        build.build()
    return pkg


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sdvg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sdvg_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_four_calls():
    syms = declared_symbols()
    for name in ("sdvg_block_attn", "sdvg_kv_commit", "sdvg_kv_rollback", "sdvg_worst_frame_route"):
        assert name in syms


def test_library_exports_every_declared_symbol(P):
    L = ctypes.CDLL(P.binding.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(L, name), name


def test_status_strings(P):
    assert P.status_string(0) == "SDVG_OK"
    for code in range(-6, 0):
        assert P.status_string(code).startswith("SDVG_ERR_")
    assert P.lib().sdvg_version() >= 100


def make_desc(P, **kw):
    d = P.binding.sdvg_attn_desc(n_q=8, n_blk=8, n_heads=2, head_dim=128,
                                 q_token_stride=256, q_head_stride=128,
                                 o_token_stride=256, o_head_stride=128,
                                 kv_token_stride=256, kv_head_stride=128,
                                 blk_token_stride=256, blk_head_stride=128,
                                 scale=128 ** -0.5, dtype=0)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


FAKE = 0x1000  # a 16-byte aligned non-null address; never dereferenced (validation fails first)


@pytest.mark.parametrize("kw,args,expect", [
    (dict(), dict(q=None), -1),
    (dict(), dict(out=None), -1),
    (dict(), dict(k_cache=None, cache_len=8), -1),
    (dict(head_dim=64), dict(), -5),
    (dict(dtype=7), dict(), -5),
    (dict(n_q=0), dict(), -2),
    (dict(n_blk=0), dict(), -2),
    (dict(n_heads=0), dict(), -2),
    (dict(q_token_stride=100), dict(), -2),
    (dict(q_token_stride=260), dict(), -4),
    (dict(kv_head_stride=132), dict(cache_len=8), -4),
    (dict(), dict(q=FAKE + 8), -4),
    (dict(), dict(cache_len=-1), -3),
    (dict(scale=-1.0), dict(), -3),
    (dict(scale=float("inf")), dict(), -3),
    (dict(scale=float("nan")), dict(), -3),
])
def test_block_attn_rejects_bad_arguments(P, kw, args, expect):
    d = make_desc(P, **kw)
    a = dict(q=FAKE, k_cache=FAKE, v_cache=FAKE, k_blk=FAKE, v_blk=FAKE, cache_len=0, out=FAKE)
    a.update(args)
    st = P.lib().sdvg_block_attn(ctypes.byref(d), a["q"], a["k_cache"], a["v_cache"], a["k_blk"],
                                 a["v_blk"], a["cache_len"], a["out"], None)
    assert st == expect, P.status_string(st)


def make_cache(P, **kw):
    c = P.binding.sdvg_kv_cache(k=FAKE, v=FAKE, n_layers=2, n_heads=2, head_dim=128, block_tokens=4,
                                capacity_tokens=12, cache_len=4, layer_stride=12 * 256,
                                token_stride=256, head_stride=128)
    for k, v in kw.items():
        setattr(c, k, v)
    return c


@pytest.mark.parametrize("kw,slot,blk,expect", [
    (dict(k=None), 1, FAKE, -1),
    (dict(), 1, None, -1),
    (dict(head_dim=64), 1, FAKE, -5),
    (dict(n_layers=0), 1, FAKE, -2),
    (dict(token_stride=257), 1, FAKE, -4),
    (dict(), 1, FAKE + 2, -4),
    (dict(), 0, FAKE, -3),      # slot already filled
    (dict(), 2, FAKE, -3),      # would leave a hole
    (dict(), -1, FAKE, -3),
    (dict(cache_len=12), 3, FAKE, -3),   # full
    (dict(cache_len=13), 1, FAKE, -3),   # inconsistent descriptor
    (dict(layer_stride=11 * 256), 1, FAKE, -2),              # a layer does not hold capacity_tokens
    (dict(token_stride=128, head_stride=128), 1, FAKE, -2),  # heads of one token overlap
    (dict(token_stride=128, head_stride=11 * 128, layer_stride=24 * 128), 1, FAKE, -2),  # head-major, head too short
    (dict(k=0x100000, layer_stride=12 * 256), 1, 0x100000 + 4 * 256 * 2, -3),        # source is the slot itself
    (dict(k=0x100000, layer_stride=12 * 256), 1, 0x100000 + 7 * 256 * 2 + 16, -3),   # source overlaps the slot's tail
    (dict(k=0x100000, v=0x200000), 1, 0x200000 + 12 * 256 * 2 + 5 * 256 * 2, -3),    # overlaps layer 1's slot of v
])
def test_kv_commit_rejects_bad_arguments(P, kw, slot, blk, expect):
    c = make_cache(P, **kw)
    before = c.cache_len
    st = P.lib().sdvg_kv_commit(ctypes.byref(c), blk, blk, slot, None)
    assert st == expect, P.status_string(st)
    assert c.cache_len == before   # state untouched on error


@pytest.mark.parametrize("new_len,expect", [(-1, -3), (5, -3), (4, 0)])
def test_kv_rollback_argument_checks(P, new_len, expect):
    c = make_cache(P)
    st = P.lib().sdvg_kv_rollback(ctypes.byref(c), new_len, None)   # new_len == cache_len: no launch
    assert st == expect
    assert c.cache_len == 4


@pytest.mark.parametrize("scores,n,tau,blk,expect", [
    (None, 12, -0.7, 1, -1), (FAKE, 0, -0.7, 1, -2), (FAKE, 12, float("nan"), 1, -3),
    (FAKE, 12, -0.7, -1, -3), (FAKE + 2, 12, -0.7, 1, -4)])
def test_route_rejects_bad_arguments(P, scores, n, tau, blk, expect):
    assert P.lib().sdvg_worst_frame_route(scores, n, tau, blk, None, None) == expect
    assert P.lib().sdvg_avg_frame_route(scores, n, tau, blk, None, None) == expect


@pytest.mark.parametrize("name", ["sdvg_worst_frame_route_batch", "sdvg_avg_frame_route_batch"])
def test_route_batch_rejects_bad_arguments(P, name):
    f = getattr(P.lib(), name)
    assert f(None, 4, 12, -0.7, None, 0, FAKE, None, None) == -1
    assert f(FAKE, 4, 12, -0.7, None, 0, None, None, None) == -1
    assert f(FAKE, 0, 12, -0.7, None, 0, FAKE, None, None) == -2
    assert f(FAKE, 4, 0, -0.7, None, 0, FAKE, None, None) == -2
    assert f(FAKE, 4, 12, float("nan"), None, 0, FAKE, None, None) == -3
    assert f(FAKE, 4, 12, -0.7, None, -2, FAKE, None, None) == -3


def test_buffer_snapshot_rejects_bad_arguments(P):
    f = P.lib().sdvg_buffer_snapshot
    assert f(None, None, 0, None) == 0                 # empty copy: nothing to do
    assert f(FAKE, FAKE + 4096, -1, None) == -2
    assert f(None, FAKE, 16, None) == -1
    assert f(FAKE, None, 16, None) == -1
    assert f(FAKE + 8, FAKE + 4096, 16, None) == -4
    assert f(FAKE, FAKE + 4096 + 4, 16, None) == -4
    assert f(FAKE, FAKE + 16, 32, None) == -3          # overlapping ranges
    assert f(FAKE + 16, FAKE, 32, None) == -3


def test_kv_descriptor_layouts_accepted(P):
    # token-major and head-major layouts that keep rows and layers apart pass validation
    # (rollback to the current length launches nothing)
    for kw in (dict(), dict(token_stride=128, head_stride=12 * 128, layer_stride=24 * 128),
               dict(n_layers=1, layer_stride=128)):
        c = make_cache(P, **kw)
        assert P.lib().sdvg_kv_rollback(ctypes.byref(c), 4, None) == 0, kw


def test_binding_checks_shapes_before_the_call(P, monkeypatch):
    """binding.block_attn rejects inconsistent tensors with ValueError before the C call (CPU
    tensors pass for the device check only because the check is patched out here)."""
    import torch
    b = P.binding
    monkeypatch.setattr(b, "_check_dev", lambda *a: None)

    class Trap:
        def __getattr__(self, name):
            raise AssertionError("the C library must not be reached")
    monkeypatch.setattr(b, "_LIB", Trap())
    bf = torch.bfloat16
    q = torch.zeros(8, 2, 128, dtype=bf)
    kb = torch.zeros(8, 2, 128, dtype=bf)
    kc = torch.zeros(16, 2, 128, dtype=bf)
    bad = [
        dict(k_cache=kc, v_cache=kc, cache_len=17),                                  # longer than the cache
        dict(k_cache=kc, v_cache=kc, cache_len=-1),
        dict(k_cache=None, v_cache=None, cache_len=4),                               # no cache given
        dict(k_cache=torch.zeros(16, 3, 128, dtype=bf), v_cache=torch.zeros(16, 3, 128, dtype=bf), cache_len=4),
        dict(k_cache=kc, v_cache=torch.zeros(12, 2, 128, dtype=bf), cache_len=4),
        dict(k_cache=kc, v_cache=kc, cache_len=4, k_blk=torch.zeros(8, 4, 128, dtype=bf)),
        dict(k_cache=kc, v_cache=kc, cache_len=4, v_blk=torch.zeros(6, 2, 128, dtype=bf)),
        dict(k_cache=kc, v_cache=kc, cache_len=4, out=torch.zeros(7, 2, 128, dtype=bf)),
        dict(k_cache=kc, v_cache=kc, cache_len=4, out=torch.zeros(8, 2, 128, dtype=torch.float32)),
        dict(k_cache=kc, v_cache=kc, cache_len=4, out=torch.zeros(8, 2, 256, dtype=bf)[:, :, ::2]),
    ]
    for kw in bad:
        args = dict(q=q, k_cache=kc, v_cache=kc, k_blk=kb, v_blk=kb, cache_len=4)
        args.update(kw)
        with pytest.raises(ValueError):
            b.block_attn(**args)


def test_rope_rejects_bad_arguments(P):
    f = P.lib().sdvg_rope
    ok = dict(x=FAKE, c=FAKE, s=FAKE, out=FAKE, n=4, H=2, d=128, xts=256, xhs=128, ots=256, ohs=128)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return f(a["x"], a["c"], a["s"], a["out"], a["n"], a["H"], a["d"], a["xts"], a["xhs"], a["ots"], a["ohs"], None)
    assert call(n=0) == 0                       # nothing to do
    assert call(n=-1) == -2 and call(H=0) == -2
    assert call(d=64) == -5
    assert call(x=None) == -1 and call(c=None) == -1 and call(out=None) == -1
    assert call(xts=100) == -2 and call(ohs=132) == -4
    assert call(x=FAKE + 2) == -4 and call(s=FAKE + 4) == -4
    g = P.lib().sdvg_kv_commit_rope
    c = make_cache(P)
    assert g(ctypes.byref(c), FAKE, FAKE, 1, None, FAKE, None) == -1
    assert g(ctypes.byref(c), FAKE, FAKE, 1, FAKE + 4, FAKE, None) == -4
    assert g(ctypes.byref(c), FAKE, FAKE, 0, FAKE, FAKE, None) == -3      # slot already filled
    assert g(ctypes.byref(c), None, FAKE, 1, FAKE, FAKE, None) == -1
    assert c.cache_len == 4


def test_fused_commit_rejects_bad_arguments(P):
    d = make_desc(P)
    f = P.lib().sdvg_block_attn_commit
    assert f(ctypes.byref(d), FAKE, None, FAKE, FAKE, FAKE, 0, FAKE, None) == -1       # needs the cache
    d.dtype = 1
    assert f(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, None) == -5       # bf16 only
    d = make_desc(P, kv_token_stride=260)
    assert f(ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, None) == -4
    c = make_cache(P)
    assert P.lib().sdvg_kv_commit_mark(ctypes.byref(c), 0) == -3 and c.cache_len == 4
    assert P.lib().sdvg_kv_commit_mark(ctypes.byref(c), 1) == 0 and c.cache_len == 8


def test_batch_rejects_bad_arguments(P):
    d = make_desc(P)
    arr = (ctypes.c_void_p * 2)(FAKE, FAKE)
    f = P.lib().sdvg_block_attn_batch
    assert f(ctypes.byref(d), 0, arr, arr, arr, arr, arr, 0, arr, None, 0, 0, None) == -2
    assert f(ctypes.byref(d), 9, arr, arr, arr, arr, arr, 0, arr, None, 0, 0, None) == -2
    assert f(ctypes.byref(d), 2, arr, arr, arr, arr, arr, 0, arr, None, -1, 0, None) == -2
    assert f(ctypes.byref(d), 2, arr, arr, arr, arr, arr, 0, arr, None, 0, 7, None) == -5
    assert f(ctypes.byref(d), 2, None, arr, arr, arr, arr, 0, arr, None, 0, 0, None) == -1
    bad = (ctypes.c_void_p * 2)(FAKE, None)
    assert f(ctypes.byref(d), 2, bad, arr, arr, arr, arr, 0, arr, None, 0, 0, None) == -1
    assert P.lib().sdvg_block_attn_workspace_bytes(ctypes.byref(d), 0, 0, 1) == -2
    assert P.lib().sdvg_block_attn_workspace_bytes(ctypes.byref(d), 1, 0, 9) == -5
    assert P.lib().sdvg_block_attn_static_workspace_limit() == 64 << 20


def test_missing_library_fails_loudly(P, monkeypatch):
    import paper_2604_17397_amd.binding as b
    monkeypatch.setattr(b, "_LIB", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libsdvg.so")
    with pytest.raises(RuntimeError):
        b.lib()
