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
#include <stddef.h>
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

// The `items` array of the kernels' single by-value AttnParams argument, read from the
// kernel-argument segment (constant memory; the compiler turns the reads into scalar loads).
__device__ __forceinline__ const sdvg::AttnItem *kernarg_items() {
  const char *ka = (const char *)__builtin_amdgcn_kernarg_segment_ptr();
  return reinterpret_cast<const sdvg::AttnItem *>(ka + offsetof(AttnParams, items));
}

// Rows of O^T held in the accumulator layout (lane = query row lane % 32, half-wave hh), scaled by
// 1 / row sum, rounded to bf16 and stored; rows past n_q are not stored.
__device__ __forceinline__ void store_rows(const AttnParams &p, const sdvg::AttnItem &it, int head, int q_row,
                                           int hh, const f32x16 (&o_acc)[4], float inv_l) {
  if (q_row >= p.n_q) return;
  uint16_t *op = static_cast<uint16_t *>(it.out) + q_row * p.o_ts + head * p.o_hs + 4 * hh;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 o4 = {o_acc[u][4 * g] * inv_l, o_acc[u][4 * g + 1] * inv_l, o_acc[u][4 * g + 2] * inv_l,
                        o_acc[u][4 * g + 3] * inv_l};
      const bf16x4 ob = __builtin_convertvector(o4, bf16x4);
      *reinterpret_cast<bf16x4 *>(op + 32 * u + 8 * g) = ob;
    }
  }
}

// Fused commit (paper Sec. 3 "Inference flow": the block the target keeps -- an accepted draft or
// its own regeneration -- goes into the target's KV cache): workgroups appended to the attention
// launch copy the block's K and V rows of this layer into cache tokens [cache_len, cache_len +
// n_blk), 16 bytes per lane, while the attention workgroups (which only read tokens below
// cache_len and the block itself) are still running. They are dispatched last and find their
// compute units among those the last round of attention workgroups leaves idle.
__device__ __forceinline__ void commit_block_rows(const AttnParams &p) {
  typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
  const sdvg::AttnItem it = kernarg_items()[0];
  const int64_t chunks = static_cast<int64_t>(p.n_blk) * p.n_heads * 16;  // 16-byte chunks per tensor
  const int64_t first = static_cast<int64_t>(blockIdx.x - p.copy_first_block) * 512 + threadIdx.x;
  const int64_t stride = static_cast<int64_t>(p.n_copy_blocks) * 512;
  auto locate = [&](int64_t g, const u32x4 *&src, u32x4 *&dst) __attribute__((always_inline)) {
    const bool is_v = g >= chunks;
    const int64_t c = is_v ? g - chunks : g;
    const int64_t row = c >> 4;
    const int ch = static_cast<int>(c & 15);
    const int64_t tok = row / p.n_heads;
    const int head = static_cast<int>(row - tok * p.n_heads);
    src = reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(is_v ? it.v_blk : it.k_blk) + tok * p.blk_ts +
                                          head * p.blk_hs + ch * 8);
    dst = reinterpret_cast<u32x4 *>(static_cast<uint16_t *>(is_v ? p.v_commit_dst : p.k_commit_dst) + tok * p.kv_ts +
                                    head * p.kv_hs + ch * 8);
  };
  // four chunks in flight per lane: the few workgroups that do this have to stream by themselves
  int64_t g = first;
  for (; g + 3 * stride < 2 * chunks; g += 4 * stride) {
    const u32x4 *s0, *s1, *s2, *s3;
    u32x4 *d0, *d1, *d2, *d3;
    locate(g, s0, d0);
    locate(g + stride, s1, d1);
    locate(g + 2 * stride, s2, d2);
    locate(g + 3 * stride, s3, d3);
    const u32x4 a = __builtin_nontemporal_load(s0), b = __builtin_nontemporal_load(s1),
                c = __builtin_nontemporal_load(s2), d = __builtin_nontemporal_load(s3);
    __builtin_nontemporal_store(a, d0);
    __builtin_nontemporal_store(b, d1);
    __builtin_nontemporal_store(c, d2);
    __builtin_nontemporal_store(d, d3);
  }
  for (; g < 2 * chunks; g += stride) {
    const u32x4 *s0;
    u32x4 *d0;
    locate(g, s0, d0);
    __builtin_nontemporal_store(__builtin_nontemporal_load(s0), d0);
  }
}

// kSplit = false: one piece per workgroup (one query tile with all its key tiles; the hot case).
// kSplit = true: the workgroup's run may hold several pieces, taken in a loop.
template <bool kSplit>
__global__ __launch_bounds__(512) void block_attn_bf16_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  char *lds_base = reinterpret_cast<char *>(smem);  // K ring at 0, V ring after it
  const uint32_t lds_addr0 =
      static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char *)lds_base));

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool group_b = wave >= 4;
  const int r32 = lane & 31;
  const int hh = lane >> 5;

  // ---- LDS read addresses (bytes)
  int k_off[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) k_off[s] = ix::k_read_offset(lane, s, 0);
  int v_off[4];
#pragma unroll
  for (int db = 0; db < 4; ++db) v_off[db] = kVBase + ix::v_read_offset(lane, 0, db, 0);

  // ---- this workgroup's run of (query tile, key tile) pairs (block_attn_index.h, "key split").
  // Normally the run is exactly one query tile with all its key tiles; when the keys are split it
  // may end one query tile and begin the next, and the loop below takes the pieces in turn.
  if (!kSplit && static_cast<int>(blockIdx.x) >= p.copy_first_block) {
    commit_block_rows(p);
    return;
  }
  const int work = ix::work_of_block(blockIdx.x, p.work_per_xcd);
  if (work >= p.total_work) return;
  int64_t u_next = static_cast<int64_t>(work) * p.units;
  const int64_t u_all = static_cast<int64_t>(p.n_hq) * p.n_tiles;
  const int64_t u_end = u_next + p.units < u_all ? u_next + p.units : u_all;
  // One piece: a query tile and a run [t_first, t_end) of its key tiles.
  auto run_piece = [&](const ix::Piece pc) __attribute__((always_inline)) {
  const int t0 = pc.t_first, t1 = pc.t_end;
  const int per_item = p.n_heads * p.n_qtiles;
  const int item = pc.hq / per_item;
  const int head = (pc.hq - item * per_item) / p.n_qtiles;
  const int qt = pc.hq - item * per_item - head * p.n_qtiles;
  // The item's pointers are read from the kernel-argument segment with a run-time index (indexing
  // the by-value parameter would first pull all items into registers).
  const sdvg::AttnItem it = kernarg_items()[item];

  // The head's 32-row wave tiles are dealt out evenly over its workgroups, so that when they do
  // not fill the last workgroup the idle waves are spread one per workgroup: every workgroup of
  // a head then streams K/V at the same pace and the re-reads stay in the XCD's L2.
  const int wt_count = ix::wave_tiles_of_qtile(qt, p.wt_base, p.wt_rem);
  const int wt_first = ix::first_wave_tile_of_qtile(qt, p.wt_base, p.wt_rem);
  const int q_row = (wt_first + wave) * 32 + r32;
  const int q_row_ld = q_row < p.n_q ? q_row : p.n_q - 1;
  bf16x8 qf[8];
  {
    const uint16_t *qp = static_cast<const uint16_t *>(it.q) + q_row_ld * p.q_ts + head * p.q_hs + 8 * hh;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }

  // ---- loader (index arithmetic in block_attn_index.h): each wave-level copy writes 1 KB of
  // LDS = 4 tile rows with the bank-conflict swizzle applied on the global side; every lane
  // keeps the global address of its two rows of the K stream and of the V stream.
  ix::Streams st;
  st.kc = reinterpret_cast<const char *>(static_cast<const uint16_t *>(it.k_cache) + head * p.kv_hs);
  st.vc = reinterpret_cast<const char *>(static_cast<const uint16_t *>(it.v_cache) + head * p.kv_hs);
  st.kb = reinterpret_cast<const char *>(static_cast<const uint16_t *>(it.k_blk) + head * p.blk_hs);
  st.vb = reinterpret_cast<const char *>(static_cast<const uint16_t *>(it.v_blk) + head * p.blk_hs);
  st.kv_tsb = static_cast<uint32_t>(p.kv_ts * 2);
  st.blk_tsb = static_cast<uint32_t>(p.blk_ts * 2);
  st.c_len = static_cast<int>(p.cache_len);
  st.n_k = p.n_k;
  const ix::Geometry geo = ix::make_geometry(st, t0, t1);
  const int n_k = p.n_k;
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
  // PV group j (0..2) with the V^T operands of step j+1 fetched into `nxt`; the last group is
  // written out in tile_body.
  auto pv_group = [&](const bf16x8(&cur)[4], bf16x8(&nxt)[4], int slot, int j)
      __attribute__((always_inline)) {
    SDVG_SB();
    read_v(nxt[0], slot, j + 1, 0);
    read_v(nxt[1], slot, j + 1, 1);
    wait_lds(N4{});
    SDVG_SB();
    mfma_v(cur[0], j, 0);
    SDVG_SB();
    read_v(nxt[2], slot, j + 1, 2);
    read_v(nxt[3], slot, j + 1, 3);
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
  cur.t_evt = ix::next_event(geo, t0);
  cur.mask_next = false;
  auto on_event = [&](int t) __attribute__((always_inline)) {
    asm volatile("" ::: "memory");  // a real branch: keep this arithmetic off the fast path
    ix::on_event(st, geo, t, wave, lane, cur);
  };

  // One tile: vector phase (softmax of S(t)), barrier, matrix phase (copies of tile t+3 started
  // between the MFMA groups, S(t+1) = K(t+1) Q^T, then O += P(t) V(t)), barrier. R = (t - t0) % 4,
  // the ring slot of tile t, is a compile-time constant: the loop is unrolled by 4 and every LDS
  // address is a base register plus an immediate.
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
    // Last PV group with the barrier ahead of its last MFMA. Everything this phase reads from LDS
    // has landed by then (the wait below), which is all the barrier stands for on this side;
    // the MFMA left over works on registers only and runs, at raised priority, while the partner
    // wave wakes up and gets its first operands ready, so the matrix pipe has work across the
    // hand-over. (More than one MFMA behind the barrier makes the vector phase the longer one.)
    SDVG_SB();
    wait_lds0();
    mfma_v(fb[0], 3, 0);
    mfma_v(fb[1], 3, 1);
    mfma_v(fb[2], 3, 2);
    SDVG_SB();
    __builtin_amdgcn_s_setprio(2);
    wg_barrier();
    SDVG_SB();
    mfma_v(fb[3], 3, 3);
    SDVG_SB();
    __builtin_amdgcn_s_setprio(0);
  };
  // ---- prologue: the piece's first three tiles into ring slots 0..2, then S of the first
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    const int t = t0 + r;
    if (t < t1) {
      if (ix::tile_is_special(geo, t)) {
        ix::row_ptrs(st, t, 0, wave, lane, cur.ptrs);
        ix::row_ptrs(st, t, 1, wave, lane, cur.ptrs);
      } else {
        ix::step_ptrs(cur.ptrs, t < geo.t_seam_lo ? geo.step_c : geo.step_b);
      }
      issue_tile(r);
    }
  }
  wait_vmcnt0();
  wg_barrier();

  if (wave >= wt_count) {
    // A wave without a wave tile computes nothing: it only keeps its share of the tile copies
    // going and takes part in the barriers, so that its SIMD is left to the partner wave.
    if (group_b) wg_barrier();
    for (int t = t0; t < t1; ++t) {
      wait_vmcnt0();
      wg_barrier();
      if (t == cur.t_evt) on_event(t);
      const int rp = (t - t0 + 3) & (kRing - 1);
#pragma unroll
      for (int i = 0; i < 4; ++i) step_copy(rp, i, cur.fast_step);
      wg_barrier();
    }
    wait_vmcnt0();
    if (!group_b) wg_barrier();
  } else {
    read_k(fa[0], 0, 0, 0);
    read_k(fa[1], 0, 0, 1);
    read_k(fa[2], 0, 1, 0);
    read_k(fa[3], 0, 1, 1);
    qk_group(fa, fb, 0, 0, 0);
    qk_group(fb, fa, 0, 1, 0);
    qk_group(fa, fb, 0, 2, 0);
    qk_group(fb, fa, 0, 3, 0);  // (its V read is harmless: slot 0 holds V of the first tile)
    wait_lds0();
    if (t0 == geo.n_tiles - 1) mask_tail(t0);
    {  // the running maximum starts at the first tile's true maximum
      const float mx = tile_max();
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s_acc[kb][i] -= mx;
      set_shift(-mx);
    }
    if (group_b) wg_barrier();  // group B runs one phase behind group A

    for (int t = t0;;) {
      tile_body(std::integral_constant<int, 0>{}, t);
      if (++t == t1) break;
      tile_body(std::integral_constant<int, 1>{}, t);
      if (++t == t1) break;
      tile_body(std::integral_constant<int, 2>{}, t);
      if (++t == t1) break;
      tile_body(std::integral_constant<int, 3>{}, t);
      if (++t == t1) break;
    }
    wait_vmcnt0();               // the redundant copies of the last tiles must not outlive the piece
    if (!group_b) wg_barrier();  // pairs with group B's extra barrier at the start

    // ---- epilogue: the finished rows, or this piece's partial sums for the merge kernel
    if (pc.whole) {
      const float inv_l = 1.0f / lane_sum32(l_run);
      store_rows(p, it, head, q_row, hh, o_acc, inv_l);
    } else {
      float *part = p.partials + static_cast<int64_t>(ix::partial_slot(pc.hq, work)) * sdvg::kPartialFloats +
                    wave * (66 * 64) + lane;
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 16; ++i) part[(16 * u + i) * 64] = o_acc[u][i];
      part[64 * 64] = l_run;
      part[65 * 64] = s_shift;
    }
  }
  };
  // A run is never longer than one query tile's key tiles, so it holds one piece or two (the end
  // of one query tile and the start of the next). Two calls rather than a loop: with the piece
  // body inside a loop the compiler kept so much alive around the back edge that it spilled.
  const ix::Piece first = ix::piece_at(u_next, u_end, p.n_tiles);
  run_piece(first);
  if (kSplit) {
    u_next += first.t_end - first.t_first;
    if (u_next < u_end) run_piece(ix::piece_at(u_next, u_end, p.n_tiles));
  }
}

// Combines the partial results of every query tile whose keys were split over several workgroups:
// with m_p the running maximum of piece p (its shift, negated) and m the largest of them,
//   O = sum_p 2^((m_p - m) scale*log2e) O_p,   l = sum_p 2^((m_p - m) scale*log2e) l_p,
// which is the same softmax as one pass over all keys (the factors only re-base the exponentials).
// One workgroup per query tile, threads laid out as in the attention kernel.
__global__ __launch_bounds__(512) void block_attn_merge_kernel(const AttnParams p) {
  const int hq = blockIdx.x;
  const int w_first = ix::first_wg_of(hq, p.n_tiles, p.units), w_last = ix::last_wg_of(hq, p.n_tiles, p.units);
  if (w_first == w_last) return;  // one workgroup had all the keys and stored the rows itself
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hh = lane >> 5;
  const int per_item = p.n_heads * p.n_qtiles;
  const int item = hq / per_item;
  const int head = (hq - item * per_item) / p.n_qtiles;
  const int qt = hq - item * per_item - head * p.n_qtiles;
  if (wave >= ix::wave_tiles_of_qtile(qt, p.wt_base, p.wt_rem)) return;
  const int q_row = (ix::first_wave_tile_of_qtile(qt, p.wt_base, p.wt_rem) + wave) * 32 + (lane & 31);
  auto part_of = [&](int w) {
    return p.partials + static_cast<int64_t>(ix::partial_slot(hq, w)) * sdvg::kPartialFloats + wave * (66 * 64) + lane;
  };
  float shift_min = part_of(w_first)[65 * 64];
  for (int w = w_first + 1; w <= w_last; ++w) shift_min = fminf(shift_min, part_of(w)[65 * 64]);
  f32x16 o_acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[u][i] = 0.f;
  float l_run = 0.f;
  for (int w = w_first; w <= w_last; ++w) {
    const float *part = part_of(w);
    const float f = __builtin_amdgcn_exp2f((shift_min - part[65 * 64]) * p.scale_log2e);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 16; ++i) o_acc[u][i] += f * part[(16 * u + i) * 64];
    l_run += f * part[64 * 64];
  }
  const float inv_l = 1.0f / lane_sum32(l_run);
  const sdvg::AttnItem it = kernarg_items()[item];
  store_rows(p, it, head, q_row, hh, o_acc, inv_l);
}

// Workspace of sdvg_block_attn_batch_static, the entry point that may not allocate: the partial
// results of a key split live in this array instead of in caller memory. Every device the
// library runs on holds its own copy, at its own address, until the process ends; host code
// never uses the array's name as an address, only the per-device pointer hipGetSymbolAddress
// returned (DeviceInfo::scratch). 64 MiB = 496 partial results of 256 rows x 128 floats (+ row
// sums and shifts): enough for every split of up to 240 query tiles over one round of 256
// workgroups (a 12-head drafter layer needs 484).
constexpr int64_t kScratchBytes = int64_t{64} << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Per-device facts the launcher needs, fetched once per device: the kernel's dynamic-LDS limit
// has to be raised (the attribute belongs to the device that is current when it is set), and the
// key split is sized by the number of compute units.
constexpr int kMaxDevices = 64;
struct DeviceInfo {
  hipError_t status = hipSuccess;
  int n_cu = 0;
  void *scratch = nullptr;  // this device's copy of the static workspace
};
int device_info(const DeviceInfo **out) {
  static std::once_flag once[kMaxDevices];
  static DeviceInfo info[kMaxDevices];
  int dev = 0;
  SDVG_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SDVG_ERR_UNSUPPORTED;
  std::call_once(once[dev], [dev] {
    constexpr size_t lds_bytes = 2 * kRing * kTileBytes;
    DeviceInfo &d = info[dev];
    d.status = hipFuncSetAttribute(reinterpret_cast<const void *>(block_attn_bf16_kernel<false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (d.status == hipSuccess)
      d.status = hipFuncSetAttribute(reinterpret_cast<const void *>(block_attn_bf16_kernel<true>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (d.status == hipSuccess)
      d.status = hipDeviceGetAttribute(&d.n_cu, hipDeviceAttributeMultiprocessorCount, dev);
    if (d.status == hipSuccess) d.status = hipGetSymbolAddress(&d.scratch, HIP_SYMBOL(scratch));
  });
  SDVG_HIP_CHECK(info[dev].status);
  *out = &info[dev];
  return SDVG_OK;
}

// How a launch is cut into workgroups. Plain: one workgroup per query tile (units == n_tiles).
// Key split: when the query tiles would leave a good part of the last round of workgroups idle
// (a drafter-shaped layer has 12 heads x 19 query tiles = 228 workgroups for 256 compute units),
// the (query tile, key tile) pairs are dealt out evenly over whole rounds instead, every
// workgroup taking the same number of pairs; query tiles cut by a workgroup boundary leave
// partial results that a second, small kernel merges.
struct Plan {
  int n_qtiles, n_hq, n_tiles, units, total_wg;
  int64_t workspace_bytes;  // 0 when nothing is split
};
Plan make_plan(int n_items, int n_q, int n_heads, int64_t n_k, int n_cu, int split_mode) {
  Plan pl;
  pl.n_qtiles = (n_q + kBM - 1) / kBM;
  pl.n_hq = n_items * n_heads * pl.n_qtiles;
  pl.n_tiles = static_cast<int>((n_k + kBN - 1) / kBN);
  pl.units = pl.n_tiles;
  pl.total_wg = pl.n_hq;
  pl.workspace_bytes = 0;
  if (split_mode == SDVG_SPLIT_NEVER || n_cu <= 0) return pl;
  const int rounds = (pl.n_hq + n_cu - 1) / n_cu;
  const double idle = 1.0 - static_cast<double>(pl.n_hq) / (static_cast<double>(rounds) * n_cu);
  // The split costs a second kernel, the partial results' traffic and a slower main kernel, and
  // a chip that is only partly busy clocks higher. Measured on MI355X (4680 queries): 12 heads
  // (11 % of the compute units idle) 15 % slower split than plain; 5 heads (63 % idle) 4 % faster;
  // 2 heads (85 % idle) 83 % faster. SDVG_SPLIT_AUTO therefore splits from 60 % idle on.
  if (pl.n_hq % n_cu == 0 || rounds > 4 || pl.n_tiles < 32) return pl;
  if (split_mode == SDVG_SPLIT_AUTO && idle < 0.6) return pl;
  const int64_t all = static_cast<int64_t>(pl.n_hq) * pl.n_tiles;
  const int64_t wgs = static_cast<int64_t>(rounds) * n_cu;
  pl.units = static_cast<int>((all + wgs - 1) / wgs);  // <= n_tiles, because wgs >= n_hq
  if (pl.units < 16) return Plan{pl.n_qtiles, pl.n_hq, pl.n_tiles, pl.n_tiles, pl.n_hq, 0};
  pl.total_wg = static_cast<int>((all + pl.units - 1) / pl.units);
  pl.workspace_bytes = static_cast<int64_t>(pl.n_hq + pl.total_wg) * sdvg::kPartialFloats * 4;
  return pl;
}

int launch_bf16(const AttnParams &p_in, const Plan &pl, int n_cu, hipStream_t s) {
  AttnParams p = p_in;
  p.n_qtiles = pl.n_qtiles;
  p.n_hq = pl.n_hq;
  p.n_tiles = pl.n_tiles;
  p.units = pl.units;
  p.total_work = pl.total_wg;
  p.work_per_xcd = (p.total_work + 7) / 8;
  const int n_wt = (p.n_q + 31) / 32;
  p.wt_base = n_wt / p.n_qtiles;
  p.wt_rem = n_wt % p.n_qtiles;
  constexpr size_t lds_bytes = 2 * kRing * kTileBytes;
  p.copy_first_block = 8 * p.work_per_xcd;
  // Fused commit: as many copying workgroups as the last round of attention workgroups leaves
  // compute units idle (they then run beside it for its whole length); a full round otherwise.
  const int idle_cus = n_cu > 0 && p.total_work % n_cu ? n_cu - p.total_work % n_cu : 0;
  p.n_copy_blocks = !p.k_commit_dst ? 0 : (idle_cus >= 4 ? idle_cus : (n_cu > 0 ? n_cu : 256));
  if (p.units == p.n_tiles)
    hipLaunchKernelGGL(block_attn_bf16_kernel<false>, dim3(8 * p.work_per_xcd + p.n_copy_blocks), dim3(512),
                       lds_bytes, s, p);
  else
    hipLaunchKernelGGL(block_attn_bf16_kernel<true>, dim3(8 * p.work_per_xcd), dim3(512), lds_bytes, s, p);
  SDVG_HIP_CHECK(hipGetLastError());
  if (p.units != p.n_tiles) {
    hipLaunchKernelGGL(block_attn_merge_kernel, dim3(p.n_hq), dim3(512), 0, s, p);
    SDVG_HIP_CHECK(hipGetLastError());
  }
  return SDVG_OK;
}

// Host-side validation shared by the entry points; fills the shape part of the parameters.
int check_desc(const sdvg_attn_desc *desc, int64_t cache_len, AttnParams &p) {
  if (!desc) return SDVG_ERR_NULL;
  if (desc->head_dim != 128) return SDVG_ERR_UNSUPPORTED;
  if (desc->dtype != SDVG_BF16 && desc->dtype != SDVG_F32) return SDVG_ERR_UNSUPPORTED;
  if (desc->n_q < 1 || desc->n_blk < 1 || desc->n_heads < 1) return SDVG_ERR_SHAPE;
  if (cache_len < 0 || cache_len + desc->n_blk > INT32_MAX) return SDVG_ERR_RANGE;
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
  }
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
  p.n_blk = desc->n_blk;
  p.n_k = static_cast<int32_t>(cache_len + desc->n_blk);
  p.n_heads = desc->n_heads;
  p.scale_log2e = scale * 1.4426950408889634f;
  return SDVG_OK;
}

int check_item(const sdvg::AttnItem &it, int64_t cache_len) {
  if (!it.q || !it.k_blk || !it.v_blk || !it.out) return SDVG_ERR_NULL;
  if (cache_len > 0 && (!it.k_cache || !it.v_cache)) return SDVG_ERR_NULL;
  if (cache_len > 0 && (!sdvg::aligned16(it.k_cache) || !sdvg::aligned16(it.v_cache))) return SDVG_ERR_ALIGN;
  if (!sdvg::aligned16(it.q) || !sdvg::aligned16(it.k_blk) || !sdvg::aligned16(it.v_blk) ||
      !sdvg::aligned16(it.out))
    return SDVG_ERR_ALIGN;
  return SDVG_OK;
}

// Common path of the batched entry points: `workspace` null means no key split.
int attn_batch(const sdvg_attn_desc *desc, int32_t n_items, const void *const *q, const void *const *k_cache,
               const void *const *v_cache, const void *const *k_blk, const void *const *v_blk,
               int64_t cache_len, void *const *out, void *workspace, int64_t workspace_bytes,
               int32_t split_mode, bool own_workspace, void *stream) {
  AttnParams p{};
  if (!desc || !q || !k_blk || !v_blk || !out) return SDVG_ERR_NULL;
  if (n_items < 1 || n_items > sdvg::kMaxAttnItems) return SDVG_ERR_SHAPE;
  if (split_mode < SDVG_SPLIT_NEVER || split_mode > SDVG_SPLIT_ALWAYS) return SDVG_ERR_UNSUPPORTED;
  int st = check_desc(desc, cache_len, p);
  if (st != SDVG_OK) return st;
  if (cache_len > 0 && (!k_cache || !v_cache)) return SDVG_ERR_NULL;
  for (int i = 0; i < n_items; ++i) {
    p.items[i] = sdvg::AttnItem{q[i], cache_len > 0 ? k_cache[i] : nullptr, cache_len > 0 ? v_cache[i] : nullptr,
                                k_blk[i], v_blk[i], out[i]};
    st = check_item(p.items[i], cache_len);
    if (st != SDVG_OK) return st;
  }
  p.n_items = n_items;
  if (desc->dtype == SDVG_F32) {  // check path: one plain launch per item
    for (int i = 0; i < n_items; ++i) {
      AttnParams one = p;
      one.items[0] = p.items[i];
      one.n_items = 1;
      st = sdvg::launch_block_attn_f32(one, static_cast<hipStream_t>(stream));
      if (st != SDVG_OK) return st;
    }
    return SDVG_OK;
  }
  if (workspace && !sdvg::aligned16(workspace)) return SDVG_ERR_ALIGN;
  const DeviceInfo *dev = nullptr;
  st = device_info(&dev);
  if (st != SDVG_OK) return st;
  if (own_workspace) {
    workspace = dev->scratch;
    workspace_bytes = kScratchBytes;
  }
  Plan pl = make_plan(n_items, p.n_q, p.n_heads, p.n_k, dev->n_cu, workspace ? split_mode : SDVG_SPLIT_NEVER);
  if (pl.workspace_bytes > workspace_bytes) {
    // the split does not fit the workspace: an error for the entry point that owns its
    // workspace (its size is a documented limit), otherwise the plain launch is always possible
    if (own_workspace) return SDVG_ERR_RANGE;
    pl = make_plan(n_items, p.n_q, p.n_heads, p.n_k, dev->n_cu, SDVG_SPLIT_NEVER);
  }
  p.partials = static_cast<float *>(workspace);
  return launch_bf16(p, pl, dev->n_cu, static_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" int sdvg_block_attn(const sdvg_attn_desc *desc, const void *q, const void *k_cache,
                               const void *v_cache, const void *k_blk, const void *v_blk,
                               int64_t cache_len, void *out, void *stream) {
  if (!desc || !q || !k_blk || !v_blk || !out) return SDVG_ERR_NULL;
  return attn_batch(desc, 1, &q, &k_cache, &v_cache, &k_blk, &v_blk, cache_len, &out, nullptr, 0, SDVG_SPLIT_NEVER,
                    false, stream);
}

extern "C" int sdvg_block_attn_commit(const sdvg_attn_desc *desc, const void *q, void *k_cache, void *v_cache,
                                      const void *k_blk, const void *v_blk, int64_t cache_len, void *out,
                                      void *stream) {
  AttnParams p{};
  if (!desc || !q || !k_blk || !v_blk || !out || !k_cache || !v_cache) return SDVG_ERR_NULL;
  if (desc->dtype != SDVG_BF16) return SDVG_ERR_UNSUPPORTED;
  int st = check_desc(desc, cache_len, p);
  if (st != SDVG_OK) return st;
  // the destination rows are addressed with the cache strides even when cache_len == 0
  if (desc->kv_token_stride < 128 || desc->kv_head_stride < 128) return SDVG_ERR_SHAPE;
  if ((desc->kv_token_stride | desc->kv_head_stride) & 7) return SDVG_ERR_ALIGN;
  if (desc->kv_token_stride >= (int64_t{1} << 30) || desc->kv_head_stride >= (int64_t{1} << 30))
    return SDVG_ERR_UNSUPPORTED;
  if (!sdvg::aligned16(k_cache) || !sdvg::aligned16(v_cache)) return SDVG_ERR_ALIGN;
  p.items[0] = sdvg::AttnItem{q, k_cache, v_cache, k_blk, v_blk, out};
  st = check_item(p.items[0], cache_len);
  if (st != SDVG_OK) return st;
  p.n_items = 1;
  p.k_commit_dst = static_cast<uint16_t *>(k_cache) + cache_len * desc->kv_token_stride;
  p.v_commit_dst = static_cast<uint16_t *>(v_cache) + cache_len * desc->kv_token_stride;
  // the block must not overlap the rows it is copied into
  const int64_t dst_bytes = ((desc->n_blk - 1) * desc->kv_token_stride + (desc->n_heads - 1) * desc->kv_head_stride + 128) * 2;
  const int64_t src_bytes = ((desc->n_blk - 1) * desc->blk_token_stride + (desc->n_heads - 1) * desc->blk_head_stride + 128) * 2;
  for (const void *src : {k_blk, v_blk})
    for (const void *dst : {static_cast<const void *>(p.k_commit_dst), static_cast<const void *>(p.v_commit_dst)}) {
      const uintptr_t a = reinterpret_cast<uintptr_t>(src), b = reinterpret_cast<uintptr_t>(dst);
      if (a < b + static_cast<uintptr_t>(dst_bytes) && b < a + static_cast<uintptr_t>(src_bytes)) return SDVG_ERR_RANGE;
    }
  const DeviceInfo *dev = nullptr;
  st = device_info(&dev);
  if (st != SDVG_OK) return st;
  const Plan pl = make_plan(1, p.n_q, p.n_heads, p.n_k, dev->n_cu, SDVG_SPLIT_NEVER);
  return launch_bf16(p, pl, dev->n_cu, static_cast<hipStream_t>(stream));
}

extern "C" int sdvg_block_attn_batch(const sdvg_attn_desc *desc, int32_t n_items, const void *const *q,
                                     const void *const *k_cache, const void *const *v_cache,
                                     const void *const *k_blk, const void *const *v_blk, int64_t cache_len,
                                     void *const *out, void *workspace, int64_t workspace_bytes,
                                     int32_t split_mode, void *stream) {
  if (workspace_bytes < 0) return SDVG_ERR_SHAPE;
  return attn_batch(desc, n_items, q, k_cache, v_cache, k_blk, v_blk, cache_len, out, workspace,
                    workspace ? workspace_bytes : 0, split_mode, false, stream);
}

extern "C" int sdvg_block_attn_batch_static(const sdvg_attn_desc *desc, int32_t n_items, const void *const *q,
                                            const void *const *k_cache, const void *const *v_cache,
                                            const void *const *k_blk, const void *const *v_blk,
                                            int64_t cache_len, void *const *out, int32_t split_mode,
                                            void *stream) {
  return attn_batch(desc, n_items, q, k_cache, v_cache, k_blk, v_blk, cache_len, out, nullptr, 0, split_mode, true,
                    stream);
}

extern "C" int64_t sdvg_block_attn_static_workspace_limit(void) { return kScratchBytes; }

extern "C" int64_t sdvg_block_attn_workspace_bytes(const sdvg_attn_desc *desc, int32_t n_items, int64_t cache_len,
                                                   int32_t split_mode) {
  AttnParams p{};
  if (n_items < 1 || n_items > sdvg::kMaxAttnItems) return SDVG_ERR_SHAPE;
  if (split_mode < SDVG_SPLIT_NEVER || split_mode > SDVG_SPLIT_ALWAYS) return SDVG_ERR_UNSUPPORTED;
  int st = check_desc(desc, cache_len, p);
  if (st != SDVG_OK) return st;
  if (desc->dtype != SDVG_BF16) return 0;
  const DeviceInfo *dev = nullptr;
  st = device_info(&dev);
  if (st != SDVG_OK) return st;
  return make_plan(n_items, p.n_q, p.n_heads, p.n_k, dev->n_cu, split_mode).workspace_bytes;
}
