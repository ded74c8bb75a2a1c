"""Host replay of the bf16 attention kernel's copy schedule (tests/host/attn_index_replay.cpp),
compiled with g++ from the same index header the kernel uses: for a dense range of
(cache_len, n_blk) and for the full-size shapes, ring tile t must hold exactly keys
64t .. 64t+63 of concat(cache, block), nothing past cache_len / n_blk is ever addressed, the read
offsets undo the copy swizzle, and the work split covers every row once. Planted mistakes in a
copy of the header must make the replay fail."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2604_17397_amd", "csrc")
REPLAY = os.path.join(ROOT, "tests", "host", "attn_index_replay.cpp")


def build(tmp_path, include_dir, name="replay"):
    exe = str(tmp_path / name)
    subprocess.run(["g++", "-O2", "-std=c++17", "-fopenmp", "-Wall", "-I", include_dir, REPLAY, "-o", exe],
                   check=True)
    return exe


def test_copy_schedule_delivers_the_concatenation(tmp_path):
    exe = build(tmp_path, CSRC)
    res = subprocess.run([exe], stdout=subprocess.PIPE, text=True, timeout=300)
    assert res.returncode == 0, res.stdout
    assert res.stdout.startswith("ok:"), res.stdout
    assert int(res.stdout.split()[1]) > 50000


MUTANTS = [
    ("event one tile late", "- kAhead;\n  g.step_c", "- kAhead + 1;\n  g.step_c"),
    ("block pitch used for the first cache steps", "return g.t_first + kAhead < g.t_seam_lo ? g.step_c : g.step_b;",
     "return g.t_first + kAhead < g.t_seam_lo ? g.step_b : g.step_c;"),
    ("second half of a wave's rows lands in the wrong place", "(i & 1) * 8 * 1024", "(i & 1) * 4 * 1024"),
    ("one pointer not re-based at an event", "  c.ptrs.v[1] -= c.fast_step;\n", ""),
    ("K swizzle dropped on the copy side", "+ row_off + (ld_p ^ (row & 15)) * 16;", "+ row_off + ld_p * 16;"),
    ("rows past the last key not clamped", "return j < s.n_k ? j : s.n_k - 1;", "return j;"),
    ("block rows addressed with the cache pitch", "* (in_cache ? s.kv_tsb : s.blk_tsb);", "* s.kv_tsb;"),
    ("seam row taken from the cache", "const bool in_cache = j < s.c_len;", "const bool in_cache = j <= s.c_len;"),
    ("V read offset without the swizzle", "((db ^ (i16 >> 2)) * 64)", "(db * 64)"),
    ("piece start ignored when the first events are looked up", "g.g_end = (g.t_ragged < g.t_end ? g.t_ragged : g.t_end) - kAhead;",
     "g.g_end = (g.t_ragged < g.n_tiles ? g.t_ragged : g.n_tiles) - kAhead;"),
    ("a piece cut at the wrong tile", "pc.t_end = left < n_tiles - pc.t_first ? pc.t_first + static_cast<int>(left) : n_tiles;",
     "pc.t_end = left < n_tiles - pc.t_first ? pc.t_first + static_cast<int>(left) + 1 : n_tiles;"),
    ("first event missed", "if (x >= g.g_lo && x <= g.g_hi) return x;", "if (x > g.g_lo && x <= g.g_hi) return x;"),
]


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_index_mistake_fails_the_replay(tmp_path, name, find, repl):
    src = open(os.path.join(CSRC, "block_attn_index.h")).read()
    assert src.count(find) == 1, "the index header changed: update this mutant's pattern"
    inc = tmp_path / "inc"
    inc.mkdir()
    (inc / "block_attn_index.h").write_text(src.replace(find, repl))
    exe = build(tmp_path, str(inc), "mutant")
    res = subprocess.run([exe], stdout=subprocess.PIPE, text=True, timeout=300)
    assert res.returncode != 0 and "FAIL" in res.stdout, name
