// Block-causal attention of one video block over the KV cache, for gfx950 (MI355X).
//
// Paper Sec. 1 / Sec. 4.1 "Models": every denoising step of a block attends to the cached keys
// and values of all previously accepted blocks plus the block itself. For one block's queries
// that is plain softmax attention over concat(cache[0:cache_len], block) with no mask.
//
// Kernel shape (bf16 path)
//   Workgroup = 8 wavefronts x 32 query rows = 256 rows of one head. Scores are computed
//   TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: the accumulator layout then gives
//   every lane one query column (col = lane % 32) and 16 keys of each 32-key half tile, so row
//   statistics are per-lane scalars, and the bf16-rounded probabilities are already in the
//   B-operand layout of the second product O^T = V^T P^T -- P never goes through LDS. Q
//   fragments stay in registers; V^T operands come from LDS with the transposing read
//   ds_read_b64_tr_b16.
//   K/V tiles of 64 keys go global -> LDS directly (global_load_lds_dwordx4, no register staging)
//   into rings of 4 K and 4 V tiles, three tiles ahead of use; bank conflicts are avoided by
//   XOR-swizzling the 16-byte chunk index with the row, applied on the global side of the copy
//   and undone on the LDS read side.
//   Ping-pong: the 8 waves form two groups (waves 0-3 and 4-7, one of each per SIMD) that run
//   half an iteration apart, so that on every SIMD one wave is in its matrix phase (S of the
//   next tile, then PV of the current one: 32 MFMAs) while the other is in its vector phase
//   (softmax of its tile). Workgroup barriers between the phases keep the groups in lockstep.
//   Softmax is in the log2 domain with a lazy running maximum whose negative is carried in the
//   initial value of the score accumulators (see softmax_tile below).
#include <math.h>
#include <stdlib.h>

#include <mutex>
#include <type_traits>

#include "block_attn_index.h"
#include "block_attn_params.h"
#include "sdvg_common.h"

namespace {

using sdvg::AttnParams;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;

namespace ix = sdvg::attn_index;
using ix::kBN;         // keys per tile
using ix::kRing;       // LDS ring depth (tiles) for K and for V
using ix::kTileBytes;  // one 64-key x 128-dim bf16 tile, unpadded
using ix::kVBase;      // the V ring follows the K ring
constexpr int kBM = 256;  // query rows per workgroup
constexpr float kPSumLimit = 1048576.0f;  // 2^20: a tile whose P sums past this retakes the maximum

// v_permlane32_swap(x, x) returns {own, partner} in the lower half-wave and {partner, own} in
// the upper one (partner = the lane 32 away); only symmetric combinations are used.
__device__ __forceinline__ float lane_max32(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float lane_sum32(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ void wait_vmcnt0() {
  // s_waitcnt vmcnt(0) only (expcnt = 7, lgkmcnt = 15 left unconstrained)
  __builtin_amdgcn_s_waitcnt(0x0F70);
}

// One wave-level 16-byte-per-lane global -> LDS copy: lane i's 16 bytes land at
// lds_addr + 16 * i. Written as inline assembly so that the compiler does not serialise
// successive copies with vmcnt(0) waits; completion is awaited explicitly (wait_vmcnt0)
// before the workgroup barrier that publishes the tile. The statements write M0 and say so in
// their clobber lists, so the compiler never assumes a value of its own survives them (clang
// warns that M0 is a reserved register it will not save; that is the intent).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, off"
      :
      : "s"(lds_addr), "v"(gptr)
      : "memory", "m0");
}
// Same copy with the 64-token pointer step folded in: the 64-bit add sits between the M0 write
// and the copy (covering the wait state M0 needs) and the stepped pointer is returned.
__device__ __forceinline__ const char *dma16_step(const char *gptr, uint64_t step, uint32_t lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %1\n\t"
      "v_lshl_add_u64 %0, %0, 0, %2\n\t"
      "global_load_lds_dwordx4 %0, off"
      : "+v"(gptr)
      : "s"(lds_addr), "s"(step)
      : "memory", "m0");
  return gptr;
}
#pragma clang diagnostic pop

// Workgroup barrier without the fence of __syncthreads (which would also wait for the
// prefetches still in flight); the compiler-level memory clobbers keep LDS accesses on
// their side of it.
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__global__ __launch_bounds__(512) void block_attn_bf16_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  char *lds_base = reinterpret_cast<char *>(smem);  // K ring at 0, V ring after it
  const uint32_t lds_addr0 =
      static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char *)lds_base));

  const int work = ix::work_of_block(blockIdx.x, p.work_per_xcd);
  if (work >= p.total_work) return;
  const int head = work / p.n_qtiles;
  const int qt = work - head * p.n_qtiles;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool group_b = wave >= 4;
  const int r32 = lane & 31;
  const int hh = lane >> 5;

  // The head's 32-row wave tiles are dealt out evenly over its workgroups, so that when they do
  // not fill the last workgroup the idle waves are spread one per workgroup: every workgroup of
  // a head then streams K/V at the same pace and the re-reads stay in the XCD's L2.
  const int wt_count = ix::wave_tiles_of_qtile(qt, p.wt_base, p.wt_rem);
  const int wt_first = ix::first_wave_tile_of_qtile(qt, p.wt_base, p.wt_rem);
  const int q_row = (wt_first + wave) * 32 + r32;
  const int q_row_ld = q_row < p.n_q ? q_row : p.n_q - 1;
  bf16x8 qf[8];
  {
    const uint16_t *qp = static_cast<const uint16_t *>(p.q) + q_row_ld * p.q_ts + head * p.q_hs + 8 * hh;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }

  // ---- loader (index arithmetic in block_attn_index.h): each wave-level copy writes 1 KB of
  // LDS = 4 tile rows with the bank-conflict swizzle applied on the global side; every lane
  // keeps the global address of its two rows of the K stream and of the V stream.
  ix::Streams st;
  st.kc = reinterpret_cast<const char *>(static_cast<const uint16_t *>(p.k_cache) + head * p.kv_hs);
  st.vc = reinterpret_cast<const char *>(static_cast<const uint16_t *>(p.v_cache) + head * p.kv_hs);
  st.kb = reinterpret_cast<const char *>(static_cast<const uint16_t *>(p.k_blk) + head * p.blk_hs);
  st.vb = reinterpret_cast<const char *>(static_cast<const uint16_t *>(p.v_blk) + head * p.blk_hs);
  st.kv_tsb = static_cast<uint32_t>(p.kv_ts * 2);
  st.blk_tsb = static_cast<uint32_t>(p.blk_ts * 2);
  st.c_len = static_cast<int>(p.cache_len);
  st.n_k = p.n_k;
  const ix::Geometry geo = ix::make_geometry(st);
  const int n_k = p.n_k;
  const int n_tiles = geo.n_tiles;
  ix::Cursor cur;
  // Starts copy number i (K rows 0-31, K rows 32-63, V rows 0-31, V rows 32-63 of this wave's
  // share) of the tile at the row pointers into ring slot `slot`.
  auto issue_tile = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16(i < 2 ? cur.ptrs.k[i] : cur.ptrs.v[i - 2], lds_addr0 + ix::copy_dst(slot, wave, i));
  };
  // Plain tiles: step the pointer by 64 tokens and start the copy in one go.
  auto step_copy = [&](int slot, int i, uint64_t step) __attribute__((always_inline)) {
    const uint32_t dst = lds_addr0 + ix::copy_dst(slot, wave, i);
    if (i < 2)
      cur.ptrs.k[i] = dma16_step(cur.ptrs.k[i], step, dst);
    else
      cur.ptrs.v[i - 2] = dma16_step(cur.ptrs.v[i - 2], step, dst);
  };

  // ---- LDS read addresses (bytes)
  int k_off[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) k_off[s] = ix::k_read_offset(lane, s, 0);
  int v_off[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) v_off[db] = kVBase + ix::v_read_offset(lane, 0, db, 0);

  f32x16 o_acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[u][i] = 0.f;
  float l_run = 0.f;
  f32x16 s_acc[2];
  bf16x8 pf[4];
  bf16x8 fa[4], fb[4];  // two groups of 4 MFMA A-operands: one in use, one being fetched
  // Minus the running maximum, in score units (before the softmax scale), and the same value in
  // all 16 registers of a score accumulator: every QK^T chain starts from it, so the scores
  // come out of the matrix cores already shifted and the softmax needs one multiply per score.
  float s_shift = 0.f;
  f32x16 s_init = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  auto set_shift = [&](float v) __attribute__((always_inline)) {
    s_shift = v;
#pragma unroll
    for (int i = 0; i < 16; ++i) s_init[i] = v;
  };

  // One V^T operand: 16 keys (step j) x dim block u, two transposing reads.
  auto read_v = [&](bf16x8 &f, int slot, int j, int u) __attribute__((always_inline)) {
    const char *vp = lds_base + v_off[u] + slot * kTileBytes + j * 16 * 256;
    const s16x4 lo =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(vp));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) s16x4 *)(vp + 8 * 256));
    const __attribute__((ext_vector_type(8))) short a16 =
        __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    __builtin_memcpy(&f, &a16, sizeof(bf16x8));
  };
  // One K operand: dim step s, 32-key half kb.
  auto read_k = [&](bf16x8 &f, int slot, int s, int kb) __attribute__((always_inline)) {
    f = *reinterpret_cast<const bf16x8 *>(lds_base + k_off[s] + slot * kTileBytes + kb * 32 * 256);
  };
  auto mfma_v = [&](const bf16x8 &f, int j, int u) __attribute__((always_inline)) {
    o_acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, pf[j], o_acc[u], 0, 0, 0);
  };
  auto mfma_k = [&](const bf16x8 &f, int s, int kb) __attribute__((always_inline)) {
    s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, qf[s], s == 0 ? s_init : s_acc[kb], 0, 0, 0);
  };
#define SDVG_SB() __builtin_amdgcn_sched_barrier(0)
  // s_waitcnt lgkmcnt(0) alone: every LDS read issued so far has returned
  auto wait_lds0 = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0xC07F); };
  // Matrix-phase building blocks. Operands come in groups of 4 (fa / fb alternate); while a
  // group's 4 MFMAs run, the next group's LDS reads are issued right after the first two MFMAs
  // (the wave would otherwise just wait for the matrix pipe), so they have two MFMA times to
  // land. K group g = dim steps 2g, 2g+1 for both key halves, operand index 2*(s&1) + kb.
  // s_waitcnt lgkmcnt(N) alone: all but the N most recent LDS reads have returned
  auto wait_lds = [&](auto n_c) __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0xC07F | (decltype(n_c)::value << 8));
  };
  using N0 = std::integral_constant<int, 0>;
  using N2 = std::integral_constant<int, 2>;
  using N4 = std::integral_constant<int, 4>;
  // QK group g; K group g+1 (or, after the last group, V group 0 of slot vslot) goes into `nxt`.
  // Half of the next group's reads are issued before this group's first MFMA (the matrix pipe
  // is still busy with the previous group's last one), the other half right after it, so every
  // operand has at least three MFMA times to arrive. Copy number g of the tile three ahead
  // (ring slot cp_slot, 64-token step cp_step) is started behind the second MFMA: no gap between
  // two MFMAs then holds more than three other instructions, which the 32 cycles of an MFMA hide.
  auto qk_group = [&](const bf16x8(&cur)[4], bf16x8(&nxt)[4], int kslot, int g, int vslot,
                      int cp_slot = -1, uint64_t cp_step = 0) __attribute__((always_inline)) {
    SDVG_SB();
    if (g < 3) {
      read_k(nxt[0], kslot, 2 * g + 2, 0);
      read_k(nxt[1], kslot, 2 * g + 2, 1);
      wait_lds(N2{});  // this group's operands have landed
    } else {
      read_v(nxt[0], vslot, 0, 0);
      read_v(nxt[1], vslot, 0, 1);
      wait_lds(N4{});
    }
    SDVG_SB();
    mfma_k(cur[0], 2 * g, 0);
    SDVG_SB();
    if (g < 3) {
      read_k(nxt[2], kslot, 2 * g + 3, 0);
      read_k(nxt[3], kslot, 2 * g + 3, 1);
    } else {
      read_v(nxt[2], vslot, 0, 2);
      read_v(nxt[3], vslot, 0, 3);
    }
    SDVG_SB();
    mfma_k(cur[1], 2 * g, 1);
    SDVG_SB();
    if (cp_slot >= 0) step_copy(cp_slot, g, cp_step);
    SDVG_SB();
    mfma_k(cur[2], 2 * g + 1, 0);
    mfma_k(cur[3], 2 * g + 1, 1);
    SDVG_SB();
  };
  // PV group j with the V^T operands of step j+1 fetched into `nxt` (none after j = 3).
  auto pv_group = [&](const bf16x8(&cur)[4], bf16x8(&nxt)[4], int slot, int j)
      __attribute__((always_inline)) {
    SDVG_SB();
    if (j < 3) {
      read_v(nxt[0], slot, j + 1, 0);
      read_v(nxt[1], slot, j + 1, 1);
      wait_lds(N4{});
    } else {
      wait_lds(N0{});
    }
    SDVG_SB();
    mfma_v(cur[0], j, 0);
    SDVG_SB();
    if (j < 3) {
      read_v(nxt[2], slot, j + 1, 2);
      read_v(nxt[3], slot, j + 1, 3);
    }
    SDVG_SB();
    mfma_v(cur[1], j, 1);
    mfma_v(cur[2], j, 2);
    mfma_v(cur[3], j, 3);
    SDVG_SB();
  };

  // Vector phase: P^T = exp2(scale*log2e * (S^T - m)) rounded to bf16 in B-operand order, plus
  // this lane's share of the row sum, taken over the ROUNDED probabilities so that numerator
  // and denominator of the softmax use the same weights. The shift by the running maximum m is
  // already in the scores (s_init), so forming P costs one multiply and one exp2 per score.
  // No maximum is computed on the fast path: m may lag the true maximum, which changes nothing
  // (both sides carry the same factor) as long as exp2 stays in range. Only if the tile's sum
  // of P comes out huge (a logit more than ~15 above m in log2 units) does the wave take the
  // slow path: raise m to the true maximum, rescale O and l, form P again.
  // The row sum unpacks the rounded pairs again (a shift and a mask) and adds them as fp32:
  // four plain instructions per pair. The one-instruction alternative, v_dot2_f32_bf16 with a
  // vector of ones, shares the matrix pipe with the partner wave's MFMAs and, queued behind
  // them at lower priority, made the vector phase the longer of the two (measured: 16 of them
  // per tile cost 250 cycles per phase; the 64 plain instructions that replace them cost none).
  // The work is laid out in stages over all 32 scores (scale, exp2, convert, sum on four
  // accumulators): no instruction depends on one issued just before it.
  auto form_p = [&]() __attribute__((always_inline)) -> float {
    float pexp[2][16];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) pexp[kb][i] = s_acc[kb][i] * p.scale_log2e;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) pexp[kb][i] = __builtin_amdgcn_exp2f(pexp[kb][i]);
    __builtin_amdgcn_sched_barrier(0);
    bf16x2 pb[2][8];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const f32x2 pp = {pexp[kb][2 * i], pexp[kb][2 * i + 1]};
        pb[kb][i] = __builtin_convertvector(pp, bf16x2);
      }
    __builtin_amdgcn_sched_barrier(0);
    float dl[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint32_t pbits;
        __builtin_memcpy(&pbits, &pb[kb][i], 4);
        const float lo = __uint_as_float(pbits << 16), hi = __uint_as_float(pbits & 0xffff0000u);
        if (kb == 0 && i < 2) {
          dl[2 * i] = lo;
          dl[2 * i + 1] = hi;
        } else {
          dl[(2 * i) & 3] += lo;
          dl[(2 * i + 1) & 3] += hi;
        }
        pf[kb * 2 + (i >> 2)][(i & 3) * 2] = pb[kb][i][0];
        pf[kb * 2 + (i >> 2)][(i & 3) * 2 + 1] = pb[kb][i][1];
      }
    __builtin_amdgcn_sched_barrier(0);
    return (dl[0] + dl[1]) + (dl[2] + dl[3]);
  };
  // Largest score of the tile for this lane's query (both half-waves), relative to the shift.
  auto tile_max = [&]() __attribute__((always_inline)) -> float {
    float m4[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) m4[c] = fmaxf(s_acc[0][c], s_acc[1][c]);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 4; i < 16; ++i) m4[i & 3] = fmaxf(m4[i & 3], s_acc[kb][i]);
    return lane_max32(fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3])));
  };
  // Moves the running maximum up by d (score units, >= 0): the scores in hand and every later
  // accumulator start d lower, and what has been summed so far shrinks by 2^(-d * scale*log2e).
  auto raise_max = [&](float d) __attribute__((always_inline)) {
    const float alpha = __builtin_amdgcn_exp2f(-d * p.scale_log2e);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 16; ++i) o_acc[u][i] *= alpha;
    l_run *= alpha;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_acc[kb][i] -= d;
    set_shift(s_shift - d);
  };
  auto softmax_tile = [&]() __attribute__((always_inline)) {
    float dl = form_p();
    if (__builtin_amdgcn_ballot_w64(!(dl < kPSumLimit)) != 0) {
      raise_max(fmaxf(tile_max(), 0.f));
      dl = form_p();
    }
    l_run += dl;
  };
  // Keys past n_k (last tile only) get -inf before the scores are shifted.
  auto mask_tail = [&](int t) __attribute__((always_inline)) {
    const int key0 = t * kBN + 4 * hh;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (key0 + kb * 32 + 8 * (i >> 2) + (i & 3) >= n_k) s_acc[kb][i] = -INFINITY;
  };

  // ---- rare events of the tile loop (block_attn_index.h, on_event): tile t starts the copies
  // of tile t+3 by stepping the row pointers 64 tokens on; where that is wrong (seam, first tile
  // wholly in the block, ragged last tile, past the end) the pointers are re-based beforehand.
  cur.fast_step = ix::first_fast_step(geo);
  cur.t_evt = ix::next_event(geo, 0);
  cur.mask_next = false;
  auto on_event = [&](int t) __attribute__((always_inline)) {
    asm volatile("" ::: "memory");  // a real branch: keep this arithmetic off the fast path
    ix::on_event(st, geo, t, wave, lane, cur);
  };

  // One tile: vector phase (softmax of S(t)), barrier, matrix phase (copies of tile t+3 started
  // between the MFMA groups, S(t+1) = K(t+1) Q^T, then O += P(t) V(t)), barrier. R = t % 4, the ring slot of tile t, is a compile-time constant: the loop is
  // unrolled by 4 and every LDS address is a base register plus an immediate.
  // The last tile computes a meaningless S(t+1) from a stale slot; nothing reads it.
  auto tile_body = [&](auto slot, int t) __attribute__((always_inline)) {
    constexpr int R = decltype(slot)::value;
    constexpr int Rn = (R + 1) % kRing;
    constexpr int Rp = (R + 3) % kRing;
    softmax_tile();
    // first operands of the matrix phase, fetched ahead of the barrier
    read_k(fa[0], Rn, 0, 0);
    read_k(fa[1], Rn, 0, 1);
    read_k(fa[2], Rn, 1, 0);
    read_k(fa[3], Rn, 1, 1);
    // keep the whole softmax on this side of the barrier
#pragma unroll
    for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(pf[j]));
    asm volatile("" : "+v"(l_run));
    wait_vmcnt0();  // this wave's copies issued in the previous matrix phase have landed
    wg_barrier();
    __builtin_amdgcn_s_setprio(1);
    if (__builtin_expect(t == cur.t_evt, 0)) on_event(t);
    // Each of the four QK groups also starts one of the four copies of tile t+3.
    qk_group(fa, fb, Rn, 0, R, Rp, cur.fast_step);
    qk_group(fb, fa, Rn, 1, R, Rp, cur.fast_step);
    qk_group(fa, fb, Rn, 2, R, Rp, cur.fast_step);
    qk_group(fb, fa, Rn, 3, R, Rp, cur.fast_step);  // leaves V group 0 in fa
    if (__builtin_expect(cur.mask_next, 0)) mask_tail(t + 1);
    pv_group(fa, fb, R, 0);
    pv_group(fb, fa, R, 1);
    pv_group(fa, fb, R, 2);
    pv_group(fb, fa, R, 3);
    // let this wave's last MFMAs retire before the partner wave takes over the matrix pipe
    asm volatile("" : "+v"(o_acc[0]), "+v"(o_acc[1]), "+v"(o_acc[2]), "+v"(o_acc[3]));
    __builtin_amdgcn_s_setprio(0);
    wg_barrier();
  };
  // ---- prologue: tiles 0..2 into the rings, then S(0)
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    if (t < n_tiles) {
      if (ix::tile_is_special(geo, t)) {
        ix::row_ptrs(st, t, 0, wave, lane, cur.ptrs);
        ix::row_ptrs(st, t, 1, wave, lane, cur.ptrs);
      } else {
        ix::step_ptrs(cur.ptrs, t < geo.t_seam_lo ? geo.step_c : geo.step_b);
      }
      issue_tile(t);
    }
  }
  wait_vmcnt0();
  wg_barrier();

  // A wave without a wave tile computes nothing: it only keeps its share of the tile copies
  // going and takes part in the barriers, so that its SIMD is left to the partner wave.
  if (wave >= wt_count) {
    if (group_b) wg_barrier();
    for (int t = 0; t < n_tiles; ++t) {
      wait_vmcnt0();
      wg_barrier();
      if (t == cur.t_evt) on_event(t);
      const int rp = (t + 3) & (kRing - 1);
#pragma unroll
      for (int i = 0; i < 4; ++i) step_copy(rp, i, cur.fast_step);
      wg_barrier();
    }
    wait_vmcnt0();
    if (!group_b) wg_barrier();
    return;
  }

  read_k(fa[0], 0, 0, 0);
  read_k(fa[1], 0, 0, 1);
  read_k(fa[2], 0, 1, 0);
  read_k(fa[3], 0, 1, 1);
  qk_group(fa, fb, 0, 0, 0);
  qk_group(fb, fa, 0, 1, 0);
  qk_group(fa, fb, 0, 2, 0);
  qk_group(fb, fa, 0, 3, 0);  // (its V read is harmless: slot 0 holds V(0))
  wait_lds0();
  if (n_tiles == 1) mask_tail(0);
  {  // the running maximum starts at tile 0's true maximum
    const float mx = tile_max();
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_acc[kb][i] -= mx;
    set_shift(-mx);
  }
  if (group_b) wg_barrier();  // group B runs one phase behind group A

  for (int t = 0;;) {
    tile_body(std::integral_constant<int, 0>{}, t);
    if (++t == n_tiles) break;
    tile_body(std::integral_constant<int, 1>{}, t);
    if (++t == n_tiles) break;
    tile_body(std::integral_constant<int, 2>{}, t);
    if (++t == n_tiles) break;
    tile_body(std::integral_constant<int, 3>{}, t);
    if (++t == n_tiles) break;
  }
  wait_vmcnt0();               // the redundant copies of the last tiles must not outlive the wave
  if (!group_b) wg_barrier();  // pairs with group B's extra barrier at the start

  // ---- epilogue
  const float l_tot = lane_sum32(l_run);
  const float inv_l = 1.0f / l_tot;
  if (q_row < p.n_q) {
    uint16_t *op = static_cast<uint16_t *>(p.out) + q_row * p.o_ts + head * p.o_hs + 4 * hh;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 o4 = {o_acc[u][4 * g] * inv_l, o_acc[u][4 * g + 1] * inv_l,
                          o_acc[u][4 * g + 2] * inv_l, o_acc[u][4 * g + 3] * inv_l};
        const bf16x4 ob = __builtin_convertvector(o4, bf16x4);
        *reinterpret_cast<bf16x4 *>(op + 32 * u + 8 * g) = ob;
      }
    }
  }
}

int launch_bf16(const AttnParams &p_in, hipStream_t s) {
  AttnParams p = p_in;
  p.n_qtiles = (p.n_q + kBM - 1) / kBM;
  const int n_wt = (p.n_q + 31) / 32;
  p.wt_base = n_wt / p.n_qtiles;
  p.wt_rem = n_wt % p.n_qtiles;
  p.total_work = p.n_qtiles * p.n_heads;
  p.work_per_xcd = (p.total_work + 7) / 8;
  constexpr size_t lds_bytes = 2 * kRing * kTileBytes;
  // The kernel needs more dynamic LDS than the default limit; the limit is raised once per
  // device (the attribute belongs to the device that is current when it is set).
  constexpr int kMaxDevices = 64;
  static std::once_flag attr_once[kMaxDevices];
  static hipError_t attr_status[kMaxDevices];
  int dev = 0;
  SDVG_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SDVG_ERR_UNSUPPORTED;
  std::call_once(attr_once[dev], [dev] {
    attr_status[dev] = hipFuncSetAttribute(reinterpret_cast<const void *>(block_attn_bf16_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
  });
  SDVG_HIP_CHECK(attr_status[dev]);
  hipLaunchKernelGGL(block_attn_bf16_kernel, dim3(8 * p.work_per_xcd), dim3(512), lds_bytes, s, p);
  SDVG_HIP_CHECK(hipGetLastError());
  return SDVG_OK;
}

}  // namespace

extern "C" int sdvg_block_attn(const sdvg_attn_desc *desc, const void *q, const void *k_cache,
                               const void *v_cache, const void *k_blk, const void *v_blk,
                               int64_t cache_len, void *out, void *stream) {
  if (!desc || !q || !k_blk || !v_blk || !out) return SDVG_ERR_NULL;
  if (desc->head_dim != 128) return SDVG_ERR_UNSUPPORTED;
  if (desc->dtype != SDVG_BF16 && desc->dtype != SDVG_F32) return SDVG_ERR_UNSUPPORTED;
  if (desc->n_q < 1 || desc->n_blk < 1 || desc->n_heads < 1) return SDVG_ERR_SHAPE;
  if (cache_len < 0 || cache_len + desc->n_blk > INT32_MAX) return SDVG_ERR_RANGE;
  if (cache_len > 0 && (!k_cache || !v_cache)) return SDVG_ERR_NULL;
  // scale == 0 selects the models' default 1/sqrt(head_dim); anything else must be finite and > 0
  if (!(desc->scale >= 0.f) || !isfinite(desc->scale)) return SDVG_ERR_RANGE;
  const float scale = desc->scale == 0.f ? 1.0f / sqrtf(static_cast<float>(desc->head_dim)) : desc->scale;
  const int64_t strides[] = {desc->q_token_stride, desc->q_head_stride, desc->o_token_stride,
                             desc->o_head_stride,  desc->blk_token_stride, desc->blk_head_stride};
  for (int64_t st : strides) {
    if (st < 128) return SDVG_ERR_SHAPE;
    if (st & 7) return SDVG_ERR_ALIGN;
    if (st >= (int64_t{1} << 30)) return SDVG_ERR_UNSUPPORTED;  // byte strides are kept in 32 bits
  }
  if (cache_len > 0) {
    if (desc->kv_token_stride < 128 || desc->kv_head_stride < 128) return SDVG_ERR_SHAPE;
    if ((desc->kv_token_stride | desc->kv_head_stride) & 7) return SDVG_ERR_ALIGN;
    if (desc->kv_token_stride >= (int64_t{1} << 30) || desc->kv_head_stride >= (int64_t{1} << 30))
      return SDVG_ERR_UNSUPPORTED;
    if (!sdvg::aligned16(k_cache) || !sdvg::aligned16(v_cache)) return SDVG_ERR_ALIGN;
  }
  if (!sdvg::aligned16(q) || !sdvg::aligned16(k_blk) || !sdvg::aligned16(v_blk) ||
      !sdvg::aligned16(out))
    return SDVG_ERR_ALIGN;

  AttnParams p{};
  p.q = q;
  p.k_cache = k_cache;
  p.v_cache = v_cache;
  p.k_blk = k_blk;
  p.v_blk = v_blk;
  p.out = out;
  p.q_ts = desc->q_token_stride;
  p.q_hs = desc->q_head_stride;
  p.o_ts = desc->o_token_stride;
  p.o_hs = desc->o_head_stride;
  p.kv_ts = desc->kv_token_stride;
  p.kv_hs = desc->kv_head_stride;
  p.blk_ts = desc->blk_token_stride;
  p.blk_hs = desc->blk_head_stride;
  p.cache_len = cache_len;
  p.n_q = desc->n_q;
  p.n_k = static_cast<int32_t>(cache_len + desc->n_blk);
  p.n_heads = desc->n_heads;
  p.scale_log2e = scale * 1.4426950408889634f;
  if (desc->dtype == SDVG_F32) return sdvg::launch_block_attn_f32(p, static_cast<hipStream_t>(stream));
  return launch_bf16(p, static_cast<hipStream_t>(stream));
}
