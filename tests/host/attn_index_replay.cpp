// Host replay of the bf16 attention kernel's copy schedule, built from the SAME index functions
// the kernel compiles in (paper_2604_17397_amd/csrc/block_attn_index.h). For one workgroup
// (8 waves x 64 lanes) it performs the prologue and the main loop's pointer updates and copies
// with fake base addresses, models what every 16-byte cell of the LDS rings then holds, and
// checks at each point of use that ring tile t is exactly keys 64t .. 64t+63 of
// concat(cache[0:c_len], block[0:n_blk]) (clamped at the last key), with the swizzle the read
// side expects, and that no copy ever addresses a token at or past c_len in the cache or at or
// past n_blk in the block. Exit code 0 = every configuration passed.
//
// usage: attn_index_replay            (dense range + the full-size shapes)
//        attn_index_replay c_len n_blk
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "block_attn_index.h"

namespace ix = sdvg::attn_index;

namespace {

constexpr uint64_t kSpan = uint64_t{1} << 44;   // distance between the four fake base addresses
const char *const kBase = reinterpret_cast<const char *>(uint64_t{1} << 48);

struct Cell {
  int stream = -1;  // 0 K, 1 V
  int key = -1;     // index into concat(cache, block)
  int chunk = -1;   // logical 16-byte chunk of the row (0..15)
};

struct Lds {
  Cell cell[2][ix::kRing][ix::kBN][16];  // [K or V][slot][row][physical chunk]
};

struct Failure {
  const char *what;
  int t, wave, lane, a, b;
};

// Decodes a fake global address into (stream, key, chunk); returns false if it is out of bounds.
bool decode(const ix::Streams &s, int n_blk, const char *p, int want_v, Cell &out) {
  const uint64_t off_all = static_cast<uint64_t>(p - kBase);
  const int region = static_cast<int>(off_all / kSpan);  // 0 kc, 1 vc, 2 kb, 3 vb
  const uint64_t off = off_all % kSpan;
  if (region < 0 || region > 3) return false;
  const bool is_v = region & 1, in_blk = region >= 2;
  if (static_cast<int>(is_v) != want_v) return false;
  const uint32_t pitch = in_blk ? s.blk_tsb : s.kv_tsb;
  const uint64_t tok = off / pitch, inner = off % pitch;
  if (inner >= 256 || inner % 16) return false;  // outside this head's 128 dims
  if (tok >= static_cast<uint64_t>(in_blk ? n_blk : s.c_len)) return false;  // past the valid tokens
  out.stream = is_v;
  out.key = static_cast<int>(in_blk ? s.c_len + tok : tok);
  out.chunk = static_cast<int>(inner / 16);
  return true;
}

bool run_copies(const ix::Streams &s, int n_blk, int slot, int t, const ix::Cursor (&cur)[ix::kWaves][64], Lds &lds,
                Failure &f) {
  for (int w = 0; w < ix::kWaves; ++w)
    for (int lane = 0; lane < 64; ++lane)
      for (int i = 0; i < 4; ++i) {
        const char *src = i < 2 ? cur[w][lane].ptrs.k[i] : cur[w][lane].ptrs.v[i - 2];
        const uint32_t dst = ix::copy_dst(slot, w, i) + 16 * lane;
        const int is_v = dst >= static_cast<uint32_t>(ix::kVBase);
        const uint32_t in_ring = dst - (is_v ? ix::kVBase : 0);
        const int dslot = in_ring / ix::kTileBytes, row = (in_ring % ix::kTileBytes) / 256, pc = (in_ring % 256) / 16;
        Cell c;
        if (dslot != slot || is_v != (i >> 1) || !decode(s, n_blk, src, is_v, c)) {
          f = {"copy source out of bounds or wrong ring", t, w, lane, i, slot};
          return false;
        }
        lds.cell[is_v][slot][row][pc] = c;
      }
  return true;
}

bool check_tile(const ix::Streams &s, const Lds &lds, int is_v, int tile, int t_first, Failure &f) {
  const int slot = (tile - t_first) % ix::kRing;
  for (int row = 0; row < ix::kBN; ++row)
    for (int pc = 0; pc < 16; ++pc) {
      const Cell &c = lds.cell[is_v][slot][row][pc];
      const int want_chunk = is_v ? pc ^ (4 * (row & 3)) : pc ^ (row & 15);
      if (c.stream != is_v || c.key != ix::key_of_row(s, tile, row) || c.chunk != want_chunk) {
        f = {is_v ? "V tile holds the wrong rows" : "K tile holds the wrong rows", tile, row, pc, c.key, c.chunk};
        return false;
      }
    }
  return true;
}

// Replays the piece [t_first, t_end) of the key tiles (the whole range when t_end < 0).
bool replay(int c_len, int n_blk, uint32_t kv_tsb, uint32_t blk_tsb, Failure &f, int t_first = 0, int t_end = -1) {
  ix::Streams s;
  s.kc = kBase;
  s.vc = kBase + kSpan;
  s.kb = kBase + 2 * kSpan;
  s.vb = kBase + 3 * kSpan;
  s.kv_tsb = kv_tsb;
  s.blk_tsb = blk_tsb;
  s.c_len = c_len;
  s.n_k = c_len + n_blk;
  const int n_tiles_all = (c_len + n_blk + ix::kBN - 1) / ix::kBN;
  if (t_end < 0) t_end = n_tiles_all;
  const ix::Geometry g = ix::make_geometry(s, t_first, t_end);
  static thread_local Lds lds;
  lds = Lds();
  static thread_local ix::Cursor cur[ix::kWaves][64];

  // prologue: the piece's first three tiles into ring slots 0..2
  for (int t = t_first; t < t_first + 3 && t < t_end; ++t) {
    for (int w = 0; w < ix::kWaves; ++w)
      for (int lane = 0; lane < 64; ++lane) {
        if (ix::tile_is_special(g, t)) {
          ix::row_ptrs(s, t, 0, w, lane, cur[w][lane].ptrs);
          ix::row_ptrs(s, t, 1, w, lane, cur[w][lane].ptrs);
        } else {
          ix::step_ptrs(cur[w][lane].ptrs, t < g.t_seam_lo ? g.step_c : g.step_b);
        }
      }
    if (!run_copies(s, n_blk, t - t_first, t, cur, lds, f)) return false;
  }
  for (int w = 0; w < ix::kWaves; ++w)
    for (int lane = 0; lane < 64; ++lane) {
      cur[w][lane].fast_step = ix::first_fast_step(g);
      cur[w][lane].t_evt = ix::next_event(g, t_first);
      cur[w][lane].mask_next = false;
    }
  if (!check_tile(s, lds, 0, t_first, t_first, f)) return false;  // S of the first tile is computed in the prologue

  bool masked_last = false;
  for (int t = t_first; t < t_end; ++t) {
    // matrix phase of tile t: S(t+1) from K slot t+1 (meaningless after the last tile), PV from V slot t
    if (t + 1 < t_end && !check_tile(s, lds, 0, t + 1, t_first, f)) return false;
    if (!check_tile(s, lds, 1, t, t_first, f)) return false;
    for (int w = 0; w < ix::kWaves; ++w)
      for (int lane = 0; lane < 64; ++lane) {
        ix::Cursor &c = cur[w][lane];
        if (t == c.t_evt) ix::on_event(s, g, t, w, lane, c);
        ix::step_ptrs(c.ptrs, c.fast_step);
      }
    if (!run_copies(s, n_blk, (t - t_first + ix::kAhead) % ix::kRing, t, cur, lds, f)) return false;
    // the tail mask is asked for exactly when the scores of the ragged last tile are produced
    const bool want_mask = t + 1 == g.n_tiles - 1 && s.n_k % ix::kBN != 0;
    for (int w = 0; w < ix::kWaves; ++w)
      if (cur[w][0].mask_next != want_mask && t + 1 < t_end) {
        f = {"tail mask flag wrong", t, w, 0, cur[w][0].mask_next, want_mask};
        return false;
      }
    masked_last |= want_mask;
  }
  // (when the ragged tile is the piece's FIRST tile the kernel masks it in its prologue instead)
  if (t_end == g.n_tiles && t_end - t_first > 1 && (s.n_k % ix::kBN != 0) != masked_last) {
    f = {"ragged last tile never masked", g.n_tiles - 1, 0, 0, 0, 0};
    return false;
  }
  return true;
}

// The read offsets must undo the swizzle of the copies.
bool check_read_side(Failure &f) {
  for (int lane = 0; lane < 64; ++lane) {
    const int r32 = lane & 31, hh = lane >> 5, i16 = lane & 15, b16 = (lane >> 4) & 1;
    for (int kb = 0; kb < 2; ++kb)
      for (int sdim = 0; sdim < 8; ++sdim) {
        const int off = ix::k_read_offset(lane, sdim, kb);
        const int row = off / 256, pc = (off % 256) / 16;
        if (off % 16 || row != 32 * kb + r32 || (pc ^ (row & 15)) != 2 * sdim + hh) {
          f = {"K read offset", sdim, kb, lane, row, pc};
          return false;
        }
      }
    for (int j = 0; j < 4; ++j)
      for (int db = 0; db < 4; ++db)
        for (int hi = 0; hi < 2; ++hi) {
          const int off = ix::v_read_offset(lane, j, db, hi);
          const int row = off / 256, b = off % 256;
          if (row != 16 * j + 8 * hi + 4 * hh + (i16 >> 2) || ((b / 64) ^ (row & 3)) != db ||
              b % 64 != 32 * b16 + 8 * (i16 & 3)) {
            f = {"V read offset", j, db, lane, row, b};
            return false;
          }
        }
  }
  return true;
}

// Every query row belongs to exactly one (q-tile, wave), no workgroup gets more than 8 wave
// tiles, and the block -> work mapping reaches every (head, q-tile) exactly once.
bool check_work_split(Failure &f) {
  for (int n_q = 1; n_q <= 6000; n_q += (n_q < 600 ? 1 : 97)) {
    const int n_qtiles = (n_q + 255) / 256, n_wt = (n_q + 31) / 32;
    const int wt_base = n_wt / n_qtiles, wt_rem = n_wt % n_qtiles;
    int next = 0;
    for (int qt = 0; qt < n_qtiles; ++qt) {
      const int cnt = ix::wave_tiles_of_qtile(qt, wt_base, wt_rem);
      if (cnt > ix::kWaves || cnt < 1 || ix::first_wave_tile_of_qtile(qt, wt_base, wt_rem) != next) {
        f = {"wave tiles not dealt out contiguously", n_q, qt, cnt, next, 0};
        return false;
      }
      next += cnt;
    }
    if (next != n_wt) {
      f = {"wave tiles lost", n_q, next, n_wt, 0, 0};
      return false;
    }
    for (int heads : {1, 12, 40}) {
      const int total = n_qtiles * heads, per_xcd = (total + 7) / 8;
      std::vector<int> seen(8 * per_xcd, 0);
      for (int b = 0; b < 8 * per_xcd; ++b) {
        const int w = ix::work_of_block(b, per_xcd);
        if (w < 0 || w >= 8 * per_xcd || seen[w]++) {
          f = {"block -> work mapping is not a bijection", n_q, heads, b, w, 0};
          return false;
        }
      }
    }
  }
  return true;
}

// Cutting the (query tile, key tile) pairs into runs: the pieces of all workgroups tile the pair
// space exactly once, a query tile's pieces lie in workgroups first_wg_of .. last_wg_of, and no
// two pieces share a partial slot.
bool check_key_split(Failure &f) {
  for (int n_hq : {1, 5, 228, 456})
    for (int n_tiles : {1, 3, 37, 220, 512})
      for (int units : {1, 2, 7, 36, 37, 196, 219, 220, 512}) {
        if (units > n_tiles) continue;
        const int64_t all = static_cast<int64_t>(n_hq) * n_tiles;
        const int n_wg = static_cast<int>((all + units - 1) / units);
        std::vector<char> seen(all, 0);
        std::vector<char> slot_used(n_hq + n_wg, 0);
        for (int w = 0; w < n_wg; ++w) {
          int64_t u = static_cast<int64_t>(w) * units;
          const int64_t u_end = u + units < all ? u + units : all;
          int pieces = 0;
          while (u < u_end) {
            const ix::Piece pc = ix::piece_at(u, u_end, n_tiles);
            const bool ok = pc.hq >= 0 && pc.hq < n_hq && pc.t_first >= 0 && pc.t_end > pc.t_first &&
                            pc.t_end <= n_tiles && pc.whole == (pc.t_first == 0 && pc.t_end == n_tiles) &&
                            w >= ix::first_wg_of(pc.hq, n_tiles, units) && w <= ix::last_wg_of(pc.hq, n_tiles, units) &&
                            (pc.whole == (ix::first_wg_of(pc.hq, n_tiles, units) == ix::last_wg_of(pc.hq, n_tiles, units)));
            if (!ok || slot_used[ix::partial_slot(pc.hq, w)]++) {
              f = {"key split: bad piece or slot used twice", n_hq, n_tiles, units, w, pc.hq};
              return false;
            }
            for (int t = pc.t_first; t < pc.t_end; ++t)
              if (seen[static_cast<int64_t>(pc.hq) * n_tiles + t]++) {
                f = {"key split: pair handled twice", n_hq, n_tiles, units, w, t};
                return false;
              }
            u += pc.t_end - pc.t_first;
            ++pieces;
          }
          (void)pieces;
        }
        for (int64_t i = 0; i < all; ++i)
          if (!seen[i]) {
            f = {"key split: pair never handled", n_hq, n_tiles, units, static_cast<int>(i / n_tiles),
                 static_cast<int>(i % n_tiles)};
            return false;
          }
      }
  return true;
}

int report(const Failure &f, int c_len, int n_blk) {
  std::printf("FAIL c_len=%d n_blk=%d: %s (t=%d, %d, %d, %d, %d)\n", c_len, n_blk, f.what, f.t, f.wave, f.lane, f.a,
              f.b);
  return 1;
}

}  // namespace

int main(int argc, char **argv) {
  Failure f{};
  if (argc == 3) {
    const int c = std::atoi(argv[1]), n = std::atoi(argv[2]);
    if (!replay(c, n, 40 * 256, 12 * 256, f)) return report(f, c, n);
    std::printf("ok c_len=%d n_blk=%d\n", c, n);
    return 0;
  }
  if (!check_read_side(f)) return report(f, -1, -1);
  if (!check_work_split(f)) return report(f, -1, -1);
  if (!check_key_split(f)) return report(f, -1, -1);
  long n_cfg = 0;
  int bad = 0;
  // dense range: every residue of c_len and n_blk modulo the tile, up to several tiles of each;
  // different row pitches for cache and block so that a mixed-up pitch cannot go unnoticed
#pragma omp parallel for schedule(dynamic, 4) reduction(+ : n_cfg)
  for (int c = 0; c < 264; ++c)
    for (int n = 1; n <= 200; ++n) {
      Failure lf{};
      if (!replay(c, n, 40 * 256, 12 * 256, lf)) {
#pragma omp critical
        if (!bad++) report(lf, c, n);
      }
      ++n_cfg;
    }
  if (bad) return 1;
  // the full-size shapes: 0..8 cached blocks of 4680 tokens plus the block itself, and the drafter's 2
  for (int k = 0; k <= 8; ++k) {
    if (!replay(4680 * k, 4680, 40 * 256, 40 * 256, f)) return report(f, 4680 * k, 4680);
    ++n_cfg;
  }
  for (int c : {1, 63, 64, 65, 4679, 4681, 9360, 32767}) {
    for (int n : {1, 63, 64, 65, 312, 4680}) {
      if (!replay(c, n, 12 * 256, 256, f)) return report(f, c, n);
      ++n_cfg;
    }
  }
  // pieces of the key range, as the key split hands them to workgroups: every start / end
  // around the seam and the ragged end, short pieces (shorter than the ring) included
  for (int c : {0, 1, 64, 100, 200, 4680, 9360})
    for (int n : {1, 70, 312, 4680}) {
      const int nt = (c + n + ix::kBN - 1) / ix::kBN;
      for (int a = 0; a < nt; a += (nt > 40 ? 7 : 1))
        for (int len : {1, 2, 3, 4, 5, 9, 64, 196}) {
          const int b = a + len < nt ? a + len : nt;
          if (!replay(c, n, 12 * 256, 40 * 256, f, a, b)) {
            std::printf("piece [%d, %d): ", a, b);
            return report(f, c, n);
          }
          ++n_cfg;
        }
    }
  std::printf("ok: %ld configurations\n", n_cfg);
  return 0;
}
