// Index arithmetic of the bf16 block-attention kernel: which key rows a wave copies into which
// LDS bytes, when the copy stream has to be re-based (cache/block seam, ragged last tile, end of
// the keys), and where the matrix phase reads its operands. Everything here is plain integer and
// pointer arithmetic, compiled both into the kernel (block_attn.hip) and into a host program
// (tests/host/attn_index_replay.cpp) that replays the copy schedule of a whole launch and checks
// that tile t of the ring holds exactly keys 64t .. 64t+63 of concat(cache, block).
//
// Paper Sec. 1 / Sec. 4.1 "Models": the keys of one attention call are the cache's first
// cache_len tokens followed by the current block's tokens; this file is that concatenation,
// expressed as addresses.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define SDVG_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define SDVG_HD inline
#endif

namespace sdvg {
namespace attn_index {

constexpr int kBN = 64;                 // keys per tile
constexpr int kRing = 4;                // LDS ring depth (tiles) for K and for V
constexpr int kTileBytes = kBN * 256;   // one 64-key x 128-dim bf16 tile, unpadded
constexpr int kVBase = kRing * kTileBytes;  // the V ring follows the K ring
constexpr int kAhead = 3;               // tile t's matrix phase starts the copies of tile t + kAhead
constexpr int kWaves = 8;               // wavefronts per workgroup

// The two sources of one head's key/value rows and their row pitches in bytes.
struct Streams {
  const char *kc, *vc;  // cache: token j (j < c_len) is at kc + j * kv_tsb
  const char *kb, *vb;  // block: token j - c_len is at kb + (j - c_len) * blk_tsb
  uint32_t kv_tsb, blk_tsb;
  int c_len, n_k;  // cached tokens; cached + block tokens
};

// Tile numbers at which the plain "64 tokens further" copy step stops being right. A workgroup
// walks a SEGMENT [t_first, t_end) of the key tiles (the whole range 0 .. n_tiles unless the
// keys of a query tile are split over several workgroups); tile numbers are absolute.
struct Geometry {
  int n_tiles;    // ceil(n_k / 64)
  int t_first;    // first tile of the segment
  int t_end;      // one past the last tile of the segment
  int t_seam_lo;  // first tile that holds a block token
  int t_seam_hi;  // first tile wholly inside the block
  int t_ragged;   // first tile with a row past the last key (== n_tiles if none)
  int g_lo, g_hi, g_end;  // the same, as seen kAhead tiles earlier by the tile that starts the copy
  uint64_t step_c, step_b;  // 64 tokens of the cache / of the block, in bytes
};

SDVG_HD Geometry make_geometry(const Streams &s, int t_first, int t_end) {
  Geometry g;
  g.n_tiles = (s.n_k + kBN - 1) / kBN;
  g.t_first = t_first;
  g.t_end = t_end;
  g.t_seam_lo = s.c_len / kBN;
  g.t_seam_hi = (s.c_len + kBN - 1) / kBN;
  g.t_ragged = s.n_k / kBN;
  g.g_lo = g.t_seam_lo - kAhead;
  g.g_hi = g.t_seam_hi - kAhead;
  g.g_end = (g.t_ragged < g.t_end ? g.t_ragged : g.t_end) - kAhead;
  g.step_c = static_cast<uint64_t>(kBN) * s.kv_tsb;
  g.step_b = static_cast<uint64_t>(kBN) * s.blk_tsb;
  return g;
}

// Key index held by row `row` (0..63) of tile t: rows past the last key repeat it (they are
// masked to -inf in the softmax; memory past the last key is never read).
SDVG_HD int key_of_row(const Streams &s, int t, int row) {
  const int j = t * kBN + row;
  return j < s.n_k ? j : s.n_k - 1;
}

// Per-lane global addresses of the copy stream. One wave-level copy moves 1 KB = 4 tile rows:
// lane i lands at row i / 16, PHYSICAL 16-byte chunk i % 16 of that row and fetches the LOGICAL
// chunk the bank-conflict swizzle maps there (K: chunk ^ (row & 15); V: chunk ^ 4 * (row & 3)).
// A wave owns rows 4*wave .. 4*wave+3 (u = 0) and 32 + 4*wave .. (u = 1) of every tile.
struct RowPtrs {
  const char *k[2], *v[2];
};

SDVG_HD int copy_row(int wave, int lane, int u) { return 4 * (wave + kWaves * u) + (lane >> 4); }

SDVG_HD void row_ptrs(const Streams &s, int t, int u, int wave, int lane, RowPtrs &r) {
  const int row = copy_row(wave, lane, u);
  const int ld_p = lane & 15;
  const int j = key_of_row(s, t, row);
  const bool in_cache = j < s.c_len;
  const uint32_t jj = static_cast<uint32_t>(in_cache ? j : j - s.c_len);
  const uint64_t row_off = static_cast<uint64_t>(jj) * (in_cache ? s.kv_tsb : s.blk_tsb);
  r.k[u] = (in_cache ? s.kc : s.kb) + row_off + (ld_p ^ (row & 15)) * 16;
  r.v[u] = (in_cache ? s.vc : s.vb) + row_off + (ld_p ^ (4 * (row & 3))) * 16;
}

SDVG_HD void step_ptrs(RowPtrs &r, uint64_t step) {
  r.k[0] += step;
  r.k[1] += step;
  r.v[0] += step;
  r.v[1] += step;
}

// Prologue (the segment's first three tiles in order): the first tile, the seam tiles, the first
// tile wholly in the block and the ragged last tile compute the pointers from scratch; every
// other tile is one 64-token step from its predecessor.
SDVG_HD bool tile_is_special(const Geometry &g, int t) {
  return t == g.t_first || static_cast<unsigned>(t - g.t_seam_lo) <= static_cast<unsigned>(g.t_seam_hi - g.t_seam_lo) ||
         t >= g.t_ragged;
}

// Byte offset inside the workgroup's LDS of copy i (0: K rows 0-31, 1: K rows 32-63, 2: V rows
// 0-31, 3: V rows 32-63 of this wave's share) of the tile in ring slot `slot`; lane i's 16 bytes
// land at this offset + 16 * i.
SDVG_HD uint32_t copy_dst(int slot, int wave, int i) {
  return static_cast<uint32_t>(slot * kTileBytes + wave * 1024 + (i & 1) * 8 * 1024 + (i >> 1) * kVBase);
}

// The main loop: tile t starts the copies of tile t + kAhead by stepping the row pointers 64
// tokens on. That is wrong when tile t + kAhead holds the cache/block seam, is the first tile
// wholly inside the block, is the ragged last tile, or does not exist; for those t (the
// "events") the pointers are set beforehand so that the step lands on the right rows (past the
// end of the segment: on its last tile again, a harmless redundant copy). next_event(x) is the first event at or
// after tile x.
SDVG_HD int next_event(const Geometry &g, int x) {
  if (x >= g.g_lo && x <= g.g_hi) return x;
  const int e = x > g.g_end ? x : g.g_end;
  return (x < g.g_lo && g.g_lo < e) ? g.g_lo : e;
}

SDVG_HD uint64_t first_fast_step(const Geometry &g) {
  return g.t_first + kAhead < g.t_seam_lo ? g.step_c : g.step_b;
}

struct Cursor {
  RowPtrs ptrs;
  uint64_t fast_step;  // what tile t adds to the pointers before it starts its copies
  int t_evt;           // next tile at which on_event has to run
  bool mask_next;      // the scores this tile's matrix phase produces need the tail mask
};

SDVG_HD void on_event(const Streams &s, const Geometry &g, int t, int wave, int lane, Cursor &c) {
  const int tau = t + kAhead < g.t_end ? t + kAhead : g.t_end - 1;
  c.fast_step = t + kAhead >= g.t_end ? 0 : (tau + 1 < g.t_seam_lo ? g.step_c : g.step_b);
  row_ptrs(s, tau, 0, wave, lane, c.ptrs);
  row_ptrs(s, tau, 1, wave, lane, c.ptrs);
  c.ptrs.k[0] -= c.fast_step;
  c.ptrs.k[1] -= c.fast_step;
  c.ptrs.v[0] -= c.fast_step;
  c.ptrs.v[1] -= c.fast_step;
  c.mask_next = t + 1 == g.n_tiles - 1 && g.t_ragged < g.n_tiles;
  c.t_evt = next_event(g, t + 1);
}

// ---- read side. A-operand of S^T = K Q^T: lane (r32 = lane % 32, hh = lane / 32) reads the 16
// bytes holding dims 16 s + 8 hh .. + 7 of key row 32 kb + r32: byte offset inside the K tile.
SDVG_HD int k_read_offset(int lane, int s, int kb) {
  const int r32 = lane & 31, hh = lane >> 5;
  return kb * 32 * 256 + r32 * 256 + (((2 * s + hh) ^ (r32 & 15)) * 16);
}
// A-operand of O^T = V^T P^T through the transposing 8-byte read: byte offset inside the V tile
// of the piece lane reads for key step j (16 keys), dim block db (32 dims), half `hi` (keys
// +8). The piece holds dims 32 db + 16 b16 + 4 (i16 & 3) .. + 3 of key row 16 j + 8 hi + 4 hh +
// (i16 >> 2), with i16 = lane % 16, b16 = (lane / 16) % 2, hh = lane / 32.
SDVG_HD int v_read_offset(int lane, int j, int db, int hi) {
  const int i16 = lane & 15, b16 = (lane >> 4) & 1, hh = lane >> 5;
  return (16 * j + 8 * hi + 4 * hh + (i16 >> 2)) * 256 + ((db ^ (i16 >> 2)) * 64) + 32 * b16 + 8 * (i16 & 3);
}

// ---- key split. The (query tile, key tile) pairs of a launch are numbered hq * n_tiles + t and
// cut into runs of `units` pairs, one run per workgroup, so that a workgroup may finish one
// query tile's keys and begin the next one's: every workgroup then has the same amount of work
// even when the query tiles do not fill the chip's compute units evenly. units == n_tiles is the
// plain case (one workgroup per query tile). A query tile whose keys are spread over several
// workgroups gets one partial result per workgroup, in slot hq + w of the partial buffer
// (distinct for distinct (hq, w): along the runs either hq or w grows from one piece to the next).
struct Piece {
  int hq;        // query tile (item, head, q-tile flattened)
  int t_first, t_end;  // its key tiles handled here
  bool whole;    // the piece covers all key tiles: the result is final, no partial is written
};
SDVG_HD Piece piece_at(int64_t u, int64_t u_end, int n_tiles) {
  Piece pc;
  pc.hq = static_cast<int>(u / n_tiles);
  pc.t_first = static_cast<int>(u - static_cast<int64_t>(pc.hq) * n_tiles);
  const int64_t left = u_end - u;
  pc.t_end = left < n_tiles - pc.t_first ? pc.t_first + static_cast<int>(left) : n_tiles;
  pc.whole = pc.t_first == 0 && pc.t_end == n_tiles;
  return pc;
}
// First and last workgroup that hold a piece of query tile hq.
SDVG_HD int first_wg_of(int hq, int n_tiles, int units) {
  return static_cast<int>(static_cast<int64_t>(hq) * n_tiles / units);
}
SDVG_HD int last_wg_of(int hq, int n_tiles, int units) {
  return static_cast<int>((static_cast<int64_t>(hq + 1) * n_tiles - 1) / units);
}
SDVG_HD int partial_slot(int hq, int wg) { return hq + wg; }

// ---- work distribution. Workgroups are dealt round-robin to the 8 XCDs; giving XCD x the
// contiguous range [x * work_per_xcd, (x + 1) * work_per_xcd) of (head, q-tile) work keeps the
// workgroups of a head on one L2.
SDVG_HD int work_of_block(int block, int work_per_xcd) { return (block % 8) * work_per_xcd + block / 8; }
// A head's 32-row wave tiles are dealt out evenly over its q-tiles (workgroups): wt_base each,
// one more for the first wt_rem.
SDVG_HD int wave_tiles_of_qtile(int qt, int wt_base, int wt_rem) { return wt_base + (qt < wt_rem ? 1 : 0); }
SDVG_HD int first_wave_tile_of_qtile(int qt, int wt_base, int wt_rem) {
  return qt * wt_base + (qt < wt_rem ? qt : wt_rem);
}

}  // namespace attn_index
}  // namespace sdvg
