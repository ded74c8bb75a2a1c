// Block-causal attention of one video block over the KV cache, for gfx950 (MI355X).
//
// Paper Sec. 1 / Sec. 4.1 "Models": every denoising step of a block attends to the cached keys
// and values of all previously accepted blocks plus the block itself. For one block's queries
// that is plain softmax attention over concat(cache[0:cache_len], block) with no mask.
//
// Kernel shape (bf16 path)
//   workgroup = NW wavefronts, each owning 32 query rows of one head; K/V tiles of 64 keys are
//   staged through LDS (double-buffered: tile t+1 travels global -> registers -> LDS while
//   tile t is consumed). Scores are computed TRANSPOSED, S^T = K Q^T, with
//   v_mfma_f32_32x32x16_bf16: the accumulator layout then gives every lane one query column
//   (col = lane % 32) and 16 of the tile's keys, so row max / row sum / rescale are per-lane
//   scalars, and the bf16-rounded probabilities are already in the B-operand layout of the
//   second product O^T = V^T P^T -- P never goes through LDS. V^T fragments come from LDS with
//   the transposing read ds_read_b64_tr_b16.
//   Softmax is online in the log2 domain with a lazy rescale: the running maximum is only
//   raised (and O, l rescaled) when a tile's maximum exceeds it by more than 2^8, which keeps
//   exp2 arguments <= 8 and removes the rescale from almost every iteration.
#include <math.h>
#include <stdlib.h>

#include <type_traits>

#include "sdvg_common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kBN = 64;        // keys per tile
constexpr int kKStride = 136;  // LDS row stride of the K tile in elements (256 B + 16 B pad)
constexpr int kVStride = 160;  // LDS row stride of the V tile in elements (256 B + 64 B pad)
constexpr int kKTile = kBN * kKStride;
constexpr int kVTile = kBN * kVStride;
constexpr float kRescaleSlack = 8.0f;  // log2 units a tile max may exceed the running max

struct AttnParams {
  const uint16_t *q, *k_cache, *v_cache, *k_blk, *v_blk;
  uint16_t *out;
  int64_t q_ts, q_hs, o_ts, o_hs, kv_ts, kv_hs, blk_ts, blk_hs;
  int64_t cache_len;
  int32_t n_q, n_k, n_heads, n_qtiles, total_work, work_per_xcd;
  float scale_log2e;  // scale * log2(e)
};

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

template <int NW>
__global__ __launch_bounds__(NW * 64) void block_attn_bf16_kernel(const AttnParams p) {
  constexpr int kThreads = NW * 64;
  constexpr int kBM = NW * 32;
  constexpr int kChunksPerThread = (kBN * 16) / kThreads;  // 16-byte chunks of one tile per thread
  static_assert((kBN * 16) % kThreads == 0, "tile must divide evenly over the workgroup");

  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t *lds_k = smem;               // [2][kBN][kKStride]
  uint16_t *lds_v = smem + 2 * kKTile;  // [2][kBN][kVStride]

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
  // (head, q-tile) work so that all q-tiles of a head stream its K/V through one L2.
  const int work = (blockIdx.x % 8) * p.work_per_xcd + blockIdx.x / 8;
  if (work >= p.total_work) return;
  const int head = work / p.n_qtiles;
  const int qt = work - head * p.n_qtiles;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r32 = lane & 31;  // MFMA row/column index of this lane
  const int hh = lane >> 5;   // which half of the 16-wide k slice this lane feeds

  // ---- Q fragments: B operand of S^T = K Q^T, kept in registers for the whole kernel
  const int q_row = qt * kBM + wave * 32 + r32;
  const int q_row_ld = q_row < p.n_q ? q_row : p.n_q - 1;
  bf16x8 qf[8];
  {
    const uint16_t *qp = p.q + q_row_ld * p.q_ts + head * p.q_hs + 8 * hh;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }

  // ---- tile loader: thread -> (row, 16-byte chunk) of the 64 x 128 tile
  const int n_tiles = (p.n_k + kBN - 1) / kBN;
  u32x4 kreg[kChunksPerThread], vreg[kChunksPerThread];
  auto load_tile = [&](int t) {
#pragma unroll
    for (int u = 0; u < kChunksPerThread; ++u) {
      const int g = tid + u * kThreads;
      const int row = g >> 4, c = g & 15;
      int64_t j = static_cast<int64_t>(t) * kBN + row;
      j = j < p.n_k ? j : p.n_k - 1;  // never read past the last valid key; masked below
      const uint16_t *kp, *vp;
      if (j < p.cache_len) {
        const int64_t off = j * p.kv_ts + head * p.kv_hs + c * 8;
        kp = p.k_cache + off;
        vp = p.v_cache + off;
      } else {
        const int64_t off = (j - p.cache_len) * p.blk_ts + head * p.blk_hs + c * 8;
        kp = p.k_blk + off;
        vp = p.v_blk + off;
      }
      kreg[u] = *reinterpret_cast<const u32x4 *>(kp);
      vreg[u] = *reinterpret_cast<const u32x4 *>(vp);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int u = 0; u < kChunksPerThread; ++u) {
      const int g = tid + u * kThreads;
      const int row = g >> 4, c = g & 15;
      *reinterpret_cast<u32x4 *>(lds_k + buf * kKTile + row * kKStride + c * 8) = kreg[u];
      *reinterpret_cast<u32x4 *>(lds_v + buf * kVTile + row * kVStride + c * 8) = vreg[u];
    }
  };

  // ---- per-lane LDS read offsets
  // K fragment (A operand of S^T): row = key r32 of a 32-key half tile, 8 dims at 16*step + 8*hh
  const int k_rd = r32 * kKStride + 8 * hh;
  // V^T fragment (A operand of O^T = V^T P^T) through the transposing read: a 16-lane group
  // reads 4 key rows x 16 dims and each lane receives 4 keys of one dim.
  const int i16 = lane & 15, b16 = (lane >> 4) & 1;
  const int v_rd = (4 * hh + (i16 >> 2)) * kVStride + 16 * b16 + 4 * (i16 & 3);

  f32x16 o_acc[4];  // O^T: o_acc[db][i] = O[q = r32][d = 32*db + 8*(i/4) + 4*hh + i%4]
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;
  float m_run = -INFINITY;  // running maximum in log2 units (already times scale*log2e)
  float l_run = 0.f;        // this lane's share of the row sum (its 16 keys of every 32)

  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int buf = t & 1;
    const bool has_next = t + 1 < n_tiles;
    if (has_next) load_tile(t + 1);

    // ---- S^T = K Q^T for 64 keys x 32 queries
    f32x16 s_acc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_acc[kb][i] = 0.f;
    const uint16_t *kbase = lds_k + buf * kKTile + k_rd;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kbase + kb * 32 * kKStride + 16 * s);
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], s_acc[kb], 0, 0, 0);
      }
    }

    // ---- mask keys past n_k (last tile only)
    if (!has_next) {
      const int key0 = t * kBN + 4 * hh;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (key0 + kb * 32 + 8 * (i >> 2) + (i & 3) >= p.n_k) s_acc[kb][i] = -INFINITY;
    }

    // ---- tile maximum per query (lane-local, then across the two half-waves)
    float mt = s_acc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mt = fmaxf(mt, s_acc[kb][i]);
    mt = lane_max32(mt) * p.scale_log2e;

    // ---- lazy rescale: only when some query's maximum grew by more than the slack
    if (__builtin_amdgcn_ballot_w64(mt > m_run + kRescaleSlack) != 0) {
      const float m_new = fmaxf(m_run, mt);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);  // exp2(-inf) = 0 on the first tile
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;
      l_run *= alpha;
      m_run = m_new;
    }

    // ---- P^T = exp2(S^T * scale*log2e - m), rounded to bf16 in B-operand order. The row sum
    // is taken over the ROUNDED probabilities (v_dot2c_f32_bf16 against (1, 1)), so numerator
    // and denominator of the softmax use the same weights.
    bf16x8 pf[4];
    const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][i], p.scale_log2e, -m_run));
        const float p1 =
            __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][i + 1], p.scale_log2e, -m_run));
        const f32x2 pp = {p0, p1};
        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
        l_run = __builtin_amdgcn_fdot2_f32_bf16(pb, ones, l_run, false);
        pf[kb * 2 + (i >> 3)][i & 7] = pb[0];
        pf[kb * 2 + (i >> 3)][(i & 7) + 1] = pb[1];
      }
    }

    // ---- O^T += V^T P^T
    const uint16_t *vbase = lds_v + buf * kVTile + v_rd;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const uint16_t *vp = vbase + (16 * j) * kVStride + 32 * db;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(vp));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(vp + 8 * kVStride));
        const __attribute__((ext_vector_type(8))) short a16 =
            __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8 a;
        __builtin_memcpy(&a, &a16, sizeof a);
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[j], o_acc[db], 0, 0, 0);
      }
    }

    if (has_next) store_tile(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: O / l, round to bf16, store
  const float l_tot = lane_sum32(l_run);
  const float inv_l = 1.0f / l_tot;
  if (q_row < p.n_q) {
    uint16_t *op = p.out + q_row * p.o_ts + head * p.o_hs + 4 * hh;
#pragma unroll
    for (int db = 0; db < 4; ++db) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 o4 = {o_acc[db][4 * g] * inv_l, o_acc[db][4 * g + 1] * inv_l,
                          o_acc[db][4 * g + 2] * inv_l, o_acc[db][4 * g + 3] * inv_l};
        const bf16x4 ob = __builtin_convertvector(o4, bf16x4);
        *reinterpret_cast<bf16x4 *>(op + 32 * db + 8 * g) = ob;
      }
    }
  }
}


// ------------------------------------------------------------------------------------------
// Ping-pong kernel: 8 wavefronts in two groups (waves 0-3 and 4-7, one of each per SIMD) that
// run half an iteration apart, so that on every SIMD one wave is in its matrix phase
// (PV of tile t, then QK^T of tile t+1) while the other is in its vector phase (softmax of a
// tile). Workgroup barriers between the phases keep the two groups in lockstep.
// K/V tiles go global -> LDS directly (global_load_lds_dwordx4, no register staging) into a
// ring of kNBuf buffers; bank conflicts are avoided by XOR-swizzling the 16-byte chunk index
// with the row (applied on the global side of the load, undone on the LDS read side).
constexpr int kNBuf = 3;
constexpr int kTileBytes = kBN * 256;  // one 64-key x 128-dim bf16 tile, unpadded


__device__ __forceinline__ void wait_vmcnt0() {
  // s_waitcnt vmcnt(0) only (expcnt = 7, lgkmcnt = 15 left unconstrained)
  __builtin_amdgcn_s_waitcnt(0x0F70);
}

// One wave-level 16-byte-per-lane global -> LDS copy: lane i's 16 bytes land at
// lds_addr + 16 * i. Written as inline assembly so that the compiler does not serialise
// successive copies with vmcnt(0) waits; completion is awaited explicitly (wait_vmcnt0)
// before the workgroup barrier that publishes the tile.
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_addr) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, off"
      :
      : "s"(lds_addr), "v"(gptr)
      : "memory");
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
      : "memory");
  return gptr;
}

// Workgroup barrier without the fence of __syncthreads (which would also wait for the
// prefetches still in flight); the compiler-level memory clobbers keep LDS accesses on
// their side of it.
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

#ifdef SDVG_ATTN_TIMING
__device__ unsigned long long g_dbg[2 * 12 + 16];
__device__ unsigned long long g_dbg2[128];
#if SDVG_ATTN_TIMING == 3
#define TS(i) do { } while (0)
#else
#define TS(i)                                                                       \
  do {                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                              \
    asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(ts[i])::"memory"); \
    __builtin_amdgcn_sched_barrier(0);                                              \
  } while (0)
#endif
#if SDVG_ATTN_TIMING == 2
#define TSX(i) TS(i)
#else
#define TSX(i) do { } while (0)
#endif
#else
#define TS(i) do { } while (0)
#define TSX(i) do { } while (0)
#endif

template <int PRIO>
__global__ __launch_bounds__(512) void block_attn_bf16_pp_kernel(const AttnParams p) {
#ifdef SDVG_ATTN_TIMING
  unsigned long long ts[12] = {0}, acc[12] = {0};
#endif
  constexpr int kBM = 256;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  char *lds_base = reinterpret_cast<char *>(smem);  // K ring at 0, V ring after it
  constexpr int kVBase = kNBuf * kTileBytes;
  const uint32_t lds_addr0 =
      static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char *)lds_base));

  const int work = (blockIdx.x % 8) * p.work_per_xcd + blockIdx.x / 8;
  if (work >= p.total_work) return;
  const int head = work / p.n_qtiles;
  const int qt = work - head * p.n_qtiles;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool group_b = wave >= 4;
  const int r32 = lane & 31;
  const int hh = lane >> 5;

  const int q_row = qt * kBM + wave * 32 + r32;
  const int q_row_ld = q_row < p.n_q ? q_row : p.n_q - 1;
  bf16x8 qf[8];
  {
    const uint16_t *qp = p.q + q_row_ld * p.q_ts + head * p.q_hs + 8 * hh;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }

  const int n_tiles = (p.n_k + kBN - 1) / kBN;

  // ---- loader: each wave-level load writes 1 KB of LDS = 4 tile rows; lane i lands at
  // row (i / 16), physical chunk (i % 16) of that block, and fetches the logical chunk that
  // the swizzle maps there. Every lane keeps the global address of its two rows for the K
  // stream and for the V stream and advances them by 64 tokens per tile; tiles that contain the
  // cache/block seam or the end of the keys recompute them (rows past the last key are
  // clamped onto it and masked in the softmax).
  const char *kc_base = reinterpret_cast<const char *>(p.k_cache + head * p.kv_hs);
  const char *vc_base = reinterpret_cast<const char *>(p.v_cache + head * p.kv_hs);
  const char *kb_base = reinterpret_cast<const char *>(p.k_blk + head * p.blk_hs);
  const char *vb_base = reinterpret_cast<const char *>(p.v_blk + head * p.blk_hs);
  const uint32_t kv_tsb = static_cast<uint32_t>(p.kv_ts * 2), blk_tsb = static_cast<uint32_t>(p.blk_ts * 2);
  const int c_len = static_cast<int>(p.cache_len), n_k = p.n_k;
  const int ld_row_in_blk = lane >> 4, ld_p = lane & 15;
  // region of tile t: 0 = wholly inside the cache, 1 = wholly inside the block, 2 = mixed/ragged
  auto region = [&](int t) {
    const int lo = t * kBN, hi = lo + kBN - 1;
    return hi < c_len ? 0 : ((lo >= c_len && hi < n_k) ? 1 : 2);
  };
  auto row_ptr = [&](int t, int u, bool is_v) -> const char * {
    const int row = 4 * (wave + 8 * u) + ld_row_in_blk;
    int j = t * kBN + row;
    j = j < n_k ? j : n_k - 1;
    const bool in_cache = j < c_len;
    const uint32_t jj = static_cast<uint32_t>(in_cache ? j : j - c_len);
    const uint64_t row_off = static_cast<uint64_t>(jj) * (in_cache ? kv_tsb : blk_tsb);
    const int chunk = is_v ? (ld_p ^ (4 * (row & 3))) : (ld_p ^ (row & 15));
    const char *base = is_v ? (in_cache ? vc_base : vb_base) : (in_cache ? kc_base : kb_base);
    return base + row_off + chunk * 16;
  };
  const char *k_ptr[2], *v_ptr[2];
  // Moves a stream's row pointers from tile t - 1 to tile t.
  auto advance = [&](const char *(&ptr)[2], int t, bool is_v) {
    const int r = region(t);
    if (t > 0 && r != 2 && r == region(t - 1)) {
      const uint64_t step = static_cast<uint64_t>(kBN) * (r == 0 ? kv_tsb : blk_tsb);
      ptr[0] += step;
      ptr[1] += step;
    } else {
      ptr[0] = row_ptr(t, 0, is_v);
      ptr[1] = row_ptr(t, 1, is_v);
    }
  };
  auto issue_k = [&](int kbuf) {
    dma16(k_ptr[0], lds_addr0 + kbuf * kTileBytes + wave * 1024);
    dma16(k_ptr[1], lds_addr0 + kbuf * kTileBytes + (wave + 8) * 1024);
  };
  auto issue_v = [&](int vbuf) {
    dma16(v_ptr[0], lds_addr0 + kVBase + vbuf * kTileBytes + wave * 1024);
    dma16(v_ptr[1], lds_addr0 + kVBase + vbuf * kTileBytes + (wave + 8) * 1024);
  };

  // ---- LDS read addresses (bytes)
  int k_off[8];  // K fragment of step s: row r32 (+32 per half tile), chunk (2s+hh) ^ (r32 & 15)
#pragma unroll
  for (int s = 0; s < 8; ++s) k_off[s] = r32 * 256 + (((2 * s + hh) ^ (r32 & 15)) * 16);
  // V^T fragment through the transposing read: a 16-lane group reads 4 key rows x 16 dims and
  // each lane receives 4 keys of one dim. The lane addressing row k of the group (k = row & 3)
  // finds logical 32-dim block db in physical 64-byte slot db ^ k of that row.
  const int i16 = lane & 15, b16 = (lane >> 4) & 1;
  int v_off[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
    v_off[db] = kVBase + (4 * hh + (i16 >> 2)) * 256 + ((db ^ (i16 >> 2)) * 64) + 32 * b16 +
                8 * (i16 & 3);

  f32x16 o_acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[u][i] = 0.f;
  float m_run = -INFINITY;
  float l_run = 0.f;
  f32x16 s_acc[2];
  bf16x8 pf[4];
  const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};

  auto qk_tile = [&](int kbuf) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_acc[kb][i] = 0.f;
    const char *kbase = lds_base + kbuf * kTileBytes;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kbase + k_off[s] + kb * 32 * 256);
        s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], s_acc[kb], 0, 0, 0);
      }
    }
  };

  auto softmax_tile = [&](int t) {
    if (t == n_tiles - 1) {
      const int key0 = t * kBN + 4 * hh;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (key0 + kb * 32 + 8 * (i >> 2) + (i & 3) >= n_k) s_acc[kb][i] = -INFINITY;
    }
    float mt = s_acc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mt = fmaxf(mt, s_acc[kb][i]);
    mt = lane_max32(mt) * p.scale_log2e;
    if (__builtin_amdgcn_ballot_w64(mt > m_run + kRescaleSlack) != 0) {
      const float m_new = fmaxf(m_run, mt);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[u][i] *= alpha;
      l_run *= alpha;
      m_run = m_new;
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][i], p.scale_log2e, -m_run));
        const float p1 =
            __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[kb][i + 1], p.scale_log2e, -m_run));
        const f32x2 pp = {p0, p1};
        const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
        l_run = __builtin_amdgcn_fdot2_f32_bf16(pb, ones, l_run, false);
        pf[kb * 2 + (i >> 3)][i & 7] = pb[0];
        pf[kb * 2 + (i >> 3)][(i & 7) + 1] = pb[1];
      }
    }
  };

  auto pv_tile = [&](int vbuf) {
    const char *vbase = lds_base + vbuf * kTileBytes;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const char *vp = vbase + v_off[u] + j * 16 * 256;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(vp));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(vp + 8 * 256));
        const __attribute__((ext_vector_type(8))) short a16 =
            __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8 a;
        __builtin_memcpy(&a, &a16, sizeof a);
        o_acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[j], o_acc[u], 0, 0, 0);
      }
    }
  };

  // ---- prologue: K(0..2), V(0..1) into the rings, then S(0)
#pragma unroll
  for (int t = 0; t < kNBuf; ++t) {
    if (t < n_tiles) {
      advance(k_ptr, t, false);
      issue_k(t);
      if (t < kNBuf - 1) {
        advance(v_ptr, t, true);
        issue_v(t);
      }
    }
  }
  wait_vmcnt0();
  wg_barrier();
  qk_tile(0);
  if (group_b) wg_barrier();  // group B runs one phase behind group A

  int kb_cur = 0;   // ring slot of K(t)
  int vb_cur = 0;   // ring slot of V(t)
  for (int t = 0; t < n_tiles; ++t) {
    // ---- vector phase: softmax of tile t
    TS(0);
    softmax_tile(t);
    // keep the whole softmax on this side of the barrier (the compiler would otherwise sink
    // the exponentials into the matrix phase)
#pragma unroll
    for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(pf[j]));
    asm volatile("" : "+v"(l_run));
    TS(1);
    wait_vmcnt0();  // this wave's loads issued in the previous matrix phase have landed
    TS(2);
    wg_barrier();
    TS(3);

    // ---- matrix phase: prefetch, O += P(t) V(t), S(t+1) = K(t+1) Q^T
    if (PRIO) __builtin_amdgcn_s_setprio(PRIO);
    const int kb_next = kb_cur + 1 == kNBuf ? 0 : kb_cur + 1;
    const int vb_free = vb_cur == 0 ? kNBuf - 1 : vb_cur - 1;  // held V(t-1), free now
    // K(t+3) replaces K(t), V(t+2) replaces V(t-1): both buffers were last read one phase ago
    if (t + kNBuf < n_tiles) {
      advance(k_ptr, t + kNBuf, false);
      TS(8);
      issue_k(kb_cur);
      TS(9);
    }
    if (t + kNBuf - 1 < n_tiles) {
      advance(v_ptr, t + kNBuf - 1, true);
      TS(10);
      issue_v(vb_free);
    }
    TS(4);
    pv_tile(vb_cur);
    TS(5);
    if (t + 1 < n_tiles) qk_tile(kb_next);
    if (PRIO) __builtin_amdgcn_s_setprio(0);
    kb_cur = kb_next;
    vb_cur = vb_cur + 1 == kNBuf ? 0 : vb_cur + 1;
    TS(6);
    if (!(group_b && t == n_tiles - 1)) wg_barrier();
    TS(7);
#ifdef SDVG_ATTN_TIMING
    if (t >= 100 && t < 164) {
      for (int i = 0; i < 7; ++i) acc[i] += ts[i + 1] - ts[i];
      acc[7] += ts[8] - ts[3];   // advance K
      acc[8] += ts[9] - ts[8];   // issue K
      acc[9] += ts[10] - ts[9];  // advance V
      acc[10] += ts[4] - ts[10]; // issue V
    }
#endif
  }
#ifdef SDVG_ATTN_TIMING
  if (work == 0 && lane == 0 && (wave == 0 || wave == 4))
    for (int i = 0; i < 11; ++i) g_dbg[(wave / 4) * 12 + i] = acc[i];
#endif

  // ---- epilogue
  const float l_tot = lane_sum32(l_run);
  const float inv_l = 1.0f / l_tot;
  if (q_row < p.n_q) {
    uint16_t *op = p.out + q_row * p.o_ts + head * p.o_hs + 4 * hh;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int db = u;
        const f32x4 o4 = {o_acc[u][4 * g] * inv_l, o_acc[u][4 * g + 1] * inv_l,
                          o_acc[u][4 * g + 2] * inv_l, o_acc[u][4 * g + 3] * inv_l};
        const bf16x4 ob = __builtin_convertvector(o4, bf16x4);
        *reinterpret_cast<bf16x4 *>(op + 32 * db + 8 * g) = ob;
      }
    }
  }
}


// ------------------------------------------------------------------------------------------
// Ping-pong kernel, second form: rings of 4 K and 4 V tiles with compile-time slot numbers (the
// tile loop is unrolled by 4, so every LDS address is a per-lane base register plus an
// immediate), one tile index for both DMA streams, and an explicitly software-pipelined matrix
// phase: the LDS reads of the next group of 4 MFMA operands are issued before the current
// group's 4 MFMAs, and the first group is already fetched at the end of the vector phase.
constexpr int kRing = 4;
constexpr float kPSumLimit = 1048576.0f;  // 2^20: a tile whose P sums past this retakes the maximum

template <int PRIO>
__global__ __launch_bounds__(512) void block_attn_bf16_pp2_kernel(const AttnParams p) {
#ifdef SDVG_ATTN_TIMING
  unsigned long long ts[12] = {0}, acc[12] = {0};
  const unsigned long long k_t0 = clock64(), k_w0 = wall_clock64();
#endif
  constexpr int kBM = 256;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  char *lds_base = reinterpret_cast<char *>(smem);  // K ring at 0, V ring after it
  constexpr int kVBase = kRing * kTileBytes;
  const uint32_t lds_addr0 =
      static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) char *)lds_base));

  const int work = (blockIdx.x % 8) * p.work_per_xcd + blockIdx.x / 8;
  if (work >= p.total_work) return;
  const int head = work / p.n_qtiles;
  const int qt = work - head * p.n_qtiles;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool group_b = wave >= 4;
  const int r32 = lane & 31;
  const int hh = lane >> 5;

  const int q_row = qt * kBM + wave * 32 + r32;
  const int q_row_ld = q_row < p.n_q ? q_row : p.n_q - 1;
  bf16x8 qf[8];
  {
    const uint16_t *qp = p.q + q_row_ld * p.q_ts + head * p.q_hs + 8 * hh;
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
  }

  const int n_k = p.n_k;
  const int n_tiles = (n_k + kBN - 1) / kBN;

  // ---- loader (see the first ping-pong kernel): lane i of a wave-level copy lands at row
  // i / 16, physical chunk i % 16 of a 1 KB block and fetches the chunk the swizzle maps there.
  const char *kc_base = reinterpret_cast<const char *>(p.k_cache + head * p.kv_hs);
  const char *vc_base = reinterpret_cast<const char *>(p.v_cache + head * p.kv_hs);
  const char *kb_base = reinterpret_cast<const char *>(p.k_blk + head * p.blk_hs);
  const char *vb_base = reinterpret_cast<const char *>(p.v_blk + head * p.blk_hs);
  const uint32_t kv_tsb = static_cast<uint32_t>(p.kv_ts * 2), blk_tsb = static_cast<uint32_t>(p.blk_ts * 2);
  const int c_len = static_cast<int>(p.cache_len);
  const int ld_row_in_blk = lane >> 4, ld_p = lane & 15;
  const int t_seam_lo = c_len / kBN;              // first tile that holds a block token
  const int t_seam_hi = (c_len + kBN - 1) / kBN;  // first tile wholly inside the block
  const uint64_t step_c = static_cast<uint64_t>(kBN) * kv_tsb, step_b = static_cast<uint64_t>(kBN) * blk_tsb;
  const char *k_ptr[2], *v_ptr[2];
  auto row_ptrs = [&](int t, int u) __attribute__((always_inline)) {
    const int row = 4 * (wave + 8 * u) + ld_row_in_blk;
    int j = t * kBN + row;
    j = j < n_k ? j : n_k - 1;  // rows past the last key re-read it; masked in the softmax
    const bool in_cache = j < c_len;
    const uint32_t jj = static_cast<uint32_t>(in_cache ? j : j - c_len);
    const uint64_t row_off = static_cast<uint64_t>(jj) * (in_cache ? kv_tsb : blk_tsb);
    k_ptr[u] = (in_cache ? kc_base : kb_base) + row_off + (ld_p ^ (row & 15)) * 16;
    v_ptr[u] = (in_cache ? vc_base : vb_base) + row_off + (ld_p ^ (4 * (row & 3))) * 16;
  };
  // Moves the row pointers to tile t (called with t = 0, 1, 2, ... in order). Tiles that hold
  // the cache/block seam, the first tile wholly in the block, and the ragged last tile recompute
  // the pointers; every other tile is one 64-token step from its predecessor.
  const int t_ragged = n_k / kBN;  // first tile with a row past the last key (== n_tiles if none)
  auto advance_ptrs = [&](int t) __attribute__((always_inline)) {
    const bool special = t == 0 || static_cast<unsigned>(t - t_seam_lo) <= static_cast<unsigned>(t_seam_hi - t_seam_lo) ||
                         t >= t_ragged;
    if (__builtin_expect(special, 0)) {
      asm volatile("" ::: "memory");  // a real branch: keep the address arithmetic off the fast path
      row_ptrs(t, 0);
      row_ptrs(t, 1);
    } else {
      const uint64_t step = t < t_seam_lo ? step_c : step_b;
      k_ptr[0] += step;
      k_ptr[1] += step;
      v_ptr[0] += step;
      v_ptr[1] += step;
    }
  };
  // Starts copy number i (K rows 0-31, K rows 32-63, V rows 0-31, V rows 32-63 of this wave's
  // share) of the tile at the row pointers into ring slot `slot`.
  auto issue_copy = [&](int slot, int i) __attribute__((always_inline)) {
    const uint32_t dst = lds_addr0 + slot * kTileBytes + wave * 1024 + (i & 1) * 8 * 1024 +
                         (i >> 1) * kVBase;
    dma16(i < 2 ? k_ptr[i] : v_ptr[i - 2], dst);
  };
  auto issue_tile = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) issue_copy(slot, i);
  };
  // Plain tiles: step the pointer by 64 tokens and start the copy in one go.
  auto step_copy = [&](int slot, int i, uint64_t step) __attribute__((always_inline)) {
    const uint32_t dst = lds_addr0 + slot * kTileBytes + wave * 1024 + (i & 1) * 8 * 1024 +
                         (i >> 1) * kVBase;
    if (i < 2)
      k_ptr[i] = dma16_step(k_ptr[i], step, dst);
    else
      v_ptr[i - 2] = dma16_step(v_ptr[i - 2], step, dst);
  };

  // ---- LDS read addresses (bytes)
  int k_off[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) k_off[s] = r32 * 256 + (((2 * s + hh) ^ (r32 & 15)) * 16);
  const int i16 = lane & 15, b16 = (lane >> 4) & 1;
  int v_off[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
    v_off[db] = kVBase + (4 * hh + (i16 >> 2)) * 256 + ((db ^ (i16 >> 2)) * 64) + 32 * b16 +
                8 * (i16 & 3);

  f32x16 o_acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[u][i] = 0.f;
  float m_run = -INFINITY;
  float l_run = 0.f;
  f32x16 s_acc[2];
  bf16x8 pf[4];
  bf16x8 fa[4], fb[4];  // two groups of 4 MFMA A-operands: one in use, one being fetched
  const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // One V^T operand: 16 keys (step j) x dim block u, two transposing reads.
  auto read_v = [&](bf16x8 &f, int slot, int j, int u) __attribute__((always_inline)) {
#ifdef SDVG_ABL_NOVREAD
    if (j > 0) { f = qf[u]; return; }
#endif
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
#ifdef SDVG_ABL_NOKREAD
    if (s > 1) { f = qf[s]; return; }
#endif
    f = *reinterpret_cast<const bf16x8 *>(lds_base + k_off[s] + slot * kTileBytes + kb * 32 * 256);
  };
  auto mfma_v = [&](const bf16x8 &f, int j, int u) __attribute__((always_inline)) {
#ifdef SDVG_ABL_HALFPV
    if (u & 1) { asm volatile("" :: "v"(f)); return; }
#endif
    o_acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, pf[j], o_acc[u], 0, 0, 0);
  };
  auto mfma_k = [&](const bf16x8 &f, int s, int kb) __attribute__((always_inline)) {
#ifdef SDVG_ABL_HALFQK
    if (s & 1) { asm volatile("" :: "v"(f)); return; }
#endif
    s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, qf[s], s == 0 ? zero16 : s_acc[kb], 0, 0, 0);
  };
#define SDVG_SB() __builtin_amdgcn_sched_barrier(0)
  // s_waitcnt lgkmcnt(0) alone: every LDS read issued so far has returned
  auto wait_lds0 = [&]() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0xC07F); };
  // Matrix-phase building blocks. Operands come in groups of 4 (fa / fb alternate); while a
  // group's 4 MFMAs run, the next group's LDS reads are issued right after the first two MFMAs
  // (the wave would otherwise just wait for the matrix pipe), so they have two MFMA times to
  // land. K group g = dim steps 2g, 2g+1 for both key halves, operand index 2*(s&1) + kb.
  // QK group g; K group g+1 (or, after the last group, V group 0 of slot vslot) goes into `nxt`
  auto qk_group = [&](const bf16x8(&cur)[4], bf16x8(&nxt)[4], int kslot, int g, int vslot)
      __attribute__((always_inline)) {
    SDVG_SB();
    wait_lds0();  // this group's operands (requested during the previous group) have landed
    SDVG_SB();
    mfma_k(cur[0], 2 * g, 0);
    SDVG_SB();
    if (g < 3) {
      read_k(nxt[0], kslot, 2 * g + 2, 0);
      read_k(nxt[1], kslot, 2 * g + 2, 1);
    } else {
      read_v(nxt[0], vslot, 0, 0);
      read_v(nxt[1], vslot, 0, 1);
    }
    SDVG_SB();
    mfma_k(cur[1], 2 * g, 1);
    SDVG_SB();
    if (g < 3) {
      read_k(nxt[2], kslot, 2 * g + 3, 0);
      read_k(nxt[3], kslot, 2 * g + 3, 1);
    } else {
      read_v(nxt[2], vslot, 0, 2);
      read_v(nxt[3], vslot, 0, 3);
    }
    SDVG_SB();
    mfma_k(cur[2], 2 * g + 1, 0);
    mfma_k(cur[3], 2 * g + 1, 1);
    SDVG_SB();
  };
  // x = s * scale*log2e - m, in place, for elements 2e and 2e+1 of the 32 scores of this lane
  auto shift_pair = [&](int e) __attribute__((always_inline)) {
#ifdef SDVG_ABL_NOSHIFT
    return;
#endif
    const int kb = e >> 3, i = (e & 7) * 2;
    s_acc[kb][i] = __builtin_fmaf(s_acc[kb][i], p.scale_log2e, -m_run);
    s_acc[kb][i + 1] = __builtin_fmaf(s_acc[kb][i + 1], p.scale_log2e, -m_run);
  };
  // PV group j with the V^T operands of step j+1 fetched into `nxt` (none after j = 3). With
  // `shift` the fresh scores of the next tile are moved to the log2 domain on the side: two
  // elements after each MFMA, in issue slots the wave would spend waiting for the matrix pipe.
  auto pv_group = [&](const bf16x8(&cur)[4], bf16x8(&nxt)[4], int slot, int j, bool shift)
      __attribute__((always_inline)) {
    SDVG_SB();
    wait_lds0();
    SDVG_SB();
    mfma_v(cur[0], j, 0);
    SDVG_SB();
    if (j < 3) {
      read_v(nxt[0], slot, j + 1, 0);
      read_v(nxt[1], slot, j + 1, 1);
    }
    if (shift) shift_pair(4 * j);
    SDVG_SB();
    mfma_v(cur[1], j, 1);
    SDVG_SB();
    if (j < 3) {
      read_v(nxt[2], slot, j + 1, 2);
      read_v(nxt[3], slot, j + 1, 3);
    }
    if (shift) shift_pair(4 * j + 1);
    SDVG_SB();
    mfma_v(cur[2], j, 2);
    SDVG_SB();
    if (shift) shift_pair(4 * j + 2);
    SDVG_SB();
    mfma_v(cur[3], j, 3);
    SDVG_SB();
    if (shift) shift_pair(4 * j + 3);
    SDVG_SB();
  };

  // Vector phase: P^T = exp2(S^T * scale*log2e - m) rounded to bf16 in B-operand order, plus
  // this lane's share of the row sum, taken over the ROUNDED probabilities so that numerator
  // and denominator of the softmax use the same weights.
  // No maximum is computed on the fast path: the running maximum m may lag the true one, which
  // changes nothing (both sides carry the same factor 2^-m) as long as exp2 stays in range.
  // Only if the tile's sum of P comes out huge (a logit more than ~15 above m in log2 units)
  // does the wave take the slow path: raise m to the true maximum, rescale O and l, form P again.
  // The wave issues in order and is alone on the vector ALU during this phase, so the work is
  // laid out in stages over all 32 scores (shift, exp2, convert, sum with four accumulators):
  // no instruction depends on one issued just before it.
  auto form_p = [&]() __attribute__((always_inline)) -> float {
    float pexp[2][16];
    const float neg_m = -m_run;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) pexp[kb][i] = __builtin_fmaf(s_acc[kb][i], p.scale_log2e, neg_m);
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
    float dl[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        dl[i & 3] = __builtin_amdgcn_fdot2_f32_bf16(pb[kb][i], ones, dl[i & 3], false);
        pf[kb * 2 + (i >> 2)][(i & 3) * 2] = pb[kb][i][0];
        pf[kb * 2 + (i >> 2)][(i & 3) * 2 + 1] = pb[kb][i][1];
      }
    __builtin_amdgcn_sched_barrier(0);
    return (dl[0] + dl[1]) + (dl[2] + dl[3]);
  };
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
  auto softmax_tile = [&]() __attribute__((always_inline)) {
#ifdef SDVG_ABL_NOSOFTMAX
    l_run += s_acc[0][0];
    return;
#endif
    float dl = form_p();
    if (__builtin_amdgcn_ballot_w64(!(dl < kPSumLimit)) != 0) {
      const float m_new = fmaxf(m_run, tile_max() * p.scale_log2e);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 16; ++i) o_acc[u][i] *= alpha;
      l_run *= alpha;
      m_run = m_new;
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

  // ---- rare events of the tile loop. Tile t starts the copies of tile t+3 by stepping the row
  // pointers 64 tokens on. That is wrong when tile t+3 holds the cache/block seam, is the
  // first tile wholly inside the block, is the ragged last tile, or does not exist; for those
  // t (t == t_evt) the pointers are set beforehand so that the step lands on the right rows
  // (past the end: on the last tile again, a harmless redundant copy).
  uint64_t fast_step = 3 < t_seam_lo ? step_c : step_b;
  const int g_lo = t_seam_lo - 3, g_hi = t_seam_hi - 3;
  const int g_end = (t_ragged < n_tiles ? t_ragged : n_tiles) - 3;
  auto next_event = [&](int x) __attribute__((always_inline)) -> int {
    if (x >= g_lo && x <= g_hi) return x;
    const int e = x > g_end ? x : g_end;
    return (x < g_lo && g_lo < e) ? g_lo : e;
  };
  int t_evt = next_event(0);
  bool mask_next = false;  // the scores produced by this tile's matrix phase need the tail mask
  auto on_event = [&](int t) __attribute__((always_inline)) {
    asm volatile("" ::: "memory");  // a real branch: keep this arithmetic off the fast path
    const int tau = t + 3 < n_tiles ? t + 3 : n_tiles - 1;
    fast_step = t + 3 >= n_tiles ? 0 : (tau + 1 < t_seam_lo ? step_c : step_b);
    row_ptrs(tau, 0);
    row_ptrs(tau, 1);
    k_ptr[0] -= fast_step;
    k_ptr[1] -= fast_step;
    v_ptr[0] -= fast_step;
    v_ptr[1] -= fast_step;
    mask_next = t + 1 == n_tiles - 1 && t_ragged < n_tiles;
    t_evt = next_event(t + 1);
  };

  // One tile: vector phase (softmax of the shifted S(t)), barrier, matrix phase (copies of tile
  // t+3 started, S(t+1) = K(t+1) Q^T, then O += P(t) V(t) with S(t+1) shifted on the side),
  // barrier. R = t % 4, the ring slot of tile t, is a compile-time constant: the loop is
  // unrolled by 4 and every LDS address is a base register plus an immediate.
  // The last tile computes a meaningless S(t+1) from a stale slot; nothing reads it.
#if defined(SDVG_ATTN_TIMING) && SDVG_ATTN_TIMING == 4
#define TSL(k)                                                                                   \
  do {                                                                                           \
    if (t >= 200 && t < 208) {                                                                   \
      unsigned long long now_;                                                                   \
      asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(now_)::"memory");               \
      if (lane == 0)                                                                             \
        *reinterpret_cast<unsigned long long *>(lds_base + 2 * kRing * kTileBytes + wave * 1024 + \
                                                ((t - 200) * 8 + (k)) * 8) = now_;               \
    }                                                                                            \
  } while (0)
#else
#define TSL(k) do { } while (0)
#endif
  auto tile_body = [&](auto slot, int t) __attribute__((always_inline)) {
    constexpr int R = decltype(slot)::value;
    constexpr int Rn = (R + 1) % kRing;
    constexpr int Rp = (R + 3) % kRing;
    TS(0);
    TSL(0);
    softmax_tile();
    TSL(1);
    // first operands of the matrix phase, fetched ahead of the barrier
    read_k(fa[0], Rn, 0, 0);
    read_k(fa[1], Rn, 0, 1);
    read_k(fa[2], Rn, 1, 0);
    read_k(fa[3], Rn, 1, 1);
    // keep the whole softmax on this side of the barrier
#pragma unroll
    for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(pf[j]));
    asm volatile("" : "+v"(l_run));
    TSX(1);
    TSL(2);
#ifndef SDVG_ABL_NOVMWAIT
    wait_vmcnt0();  // this wave's copies issued in the previous matrix phase have landed
#endif
    TS(2);
    TSL(3);
    wg_barrier();
    TSL(4);
    TS(3);
    if (PRIO == 1) __builtin_amdgcn_s_setprio(1);
    if (PRIO == 2) __builtin_amdgcn_s_setprio(0);
    if (__builtin_expect(t == t_evt, 0)) on_event(t);
    // After each of the first four MFMA groups one copy of tile t+3 is started: the matrix
    // pipe is still busy with the group's last MFMA, so these few instructions cost nothing.
    qk_group(fa, fb, Rn, 0, R);
#ifndef SDVG_ABL_NODMA
    step_copy(Rp, 0, fast_step);
#endif
    qk_group(fb, fa, Rn, 1, R);
#ifndef SDVG_ABL_NODMA
    step_copy(Rp, 1, fast_step);
#endif
    TSX(4);
    qk_group(fa, fb, Rn, 2, R);
#ifndef SDVG_ABL_NODMA
    step_copy(Rp, 2, fast_step);
#endif
    qk_group(fb, fa, Rn, 3, R);  // leaves V group 0 in fa
#ifndef SDVG_ABL_NODMA
    step_copy(Rp, 3, fast_step);
#endif
    if (__builtin_expect(mask_next, 0)) mask_tail(t + 1);
    TSX(5);
    TSL(5);
    pv_group(fa, fb, R, 0, false);
    pv_group(fb, fa, R, 1, false);
    pv_group(fa, fb, R, 2, false);
    pv_group(fb, fa, R, 3, false);
    if (PRIO == 1) __builtin_amdgcn_s_setprio(0);
    if (PRIO == 2) __builtin_amdgcn_s_setprio(1);
    TS(6);
    TSL(6);
#ifndef SDVG_ABL_NOBAR2
    wg_barrier();
#endif
    TSL(7);
    TS(7);
#if defined(SDVG_ATTN_TIMING) && SDVG_ATTN_TIMING != 3
    if (t >= 100 && t < 164) {
#if SDVG_ATTN_TIMING == 2
      for (int i = 0; i < 7; ++i) acc[i] += ts[i + 1] - ts[i];
#else
      acc[0] += ts[2] - ts[0];
      acc[1] += ts[3] - ts[2];
      acc[2] += ts[6] - ts[3];
      acc[3] += ts[7] - ts[6];
#endif
      acc[9] += ts[0] - ts[11];
    }
    ts[11] = ts[7];
    if ((t & 63) == 0 && work == 0 && lane == 0 && wave == 0) g_dbg[24 + (t >> 6)] = ts[0] - k_t0;
#endif
  };
  // ---- prologue: tiles 0..2 into the rings, then S(0)
#pragma unroll
  for (int t = 0; t < 3; ++t) {
    if (t < n_tiles) {
      advance_ptrs(t);
      issue_tile(t);
    }
  }
  wait_vmcnt0();
  wg_barrier();
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
  m_run = tile_max() * p.scale_log2e;  // the running maximum starts at tile 0's true maximum
#ifndef SDVG_ABL_NOBAR2
  if (group_b) wg_barrier();  // group B runs one phase behind group A
#endif

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
#ifndef SDVG_ABL_NOBAR2
  if (!group_b) wg_barrier();  // pairs with group B's extra barrier at the start
#endif
#if defined(SDVG_ATTN_TIMING) && SDVG_ATTN_TIMING == 4
  __syncthreads();
  if (work == 0 && lane == 0 && (wave == 0 || wave == 4))
    for (int i = 0; i < 64; ++i)
      g_dbg2[(wave / 4) * 64 + i] = *reinterpret_cast<unsigned long long *>(
          lds_base + 2 * kRing * kTileBytes + wave * 1024 + i * 8);
#endif
#ifdef SDVG_ATTN_TIMING
  if (work == 0 && lane == 0 && (wave == 0 || wave == 4))
  {
    acc[7] = clock64() - k_t0;
    acc[8] = wall_clock64() - k_w0;
    for (int i = 0; i < 11; ++i) g_dbg[(wave / 4) * 12 + i] = acc[i];
  }
#endif

  // ---- epilogue
  const float l_tot = lane_sum32(l_run);
  const float inv_l = 1.0f / l_tot;
  if (q_row < p.n_q) {
    uint16_t *op = p.out + q_row * p.o_ts + head * p.o_hs + 4 * hh;
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

template <int PRIO>
int launch_bf16_pp2(const AttnParams &p_in, hipStream_t s) {
  AttnParams p = p_in;
  p.n_qtiles = (p.n_q + 255) / 256;
  p.total_work = p.n_qtiles * p.n_heads;
  p.work_per_xcd = (p.total_work + 7) / 8;
#if defined(SDVG_ATTN_TIMING) && SDVG_ATTN_TIMING == 4
  constexpr size_t lds_bytes = 2 * kRing * kTileBytes + 8192;
#else
  constexpr size_t lds_bytes = 2 * kRing * kTileBytes;
#endif
  static bool attr_set = false;
  if (!attr_set) {
    SDVG_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(block_attn_bf16_pp2_kernel<PRIO>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    attr_set = true;
  }
  hipLaunchKernelGGL(block_attn_bf16_pp2_kernel<PRIO>, dim3(8 * p.work_per_xcd), dim3(512), lds_bytes,
                     s, p);
  SDVG_HIP_CHECK(hipGetLastError());
  return SDVG_OK;
}

template <int PRIO>
int launch_bf16_pp(const AttnParams &p_in, hipStream_t s) {
  AttnParams p = p_in;
  p.n_qtiles = (p.n_q + 255) / 256;
  p.total_work = p.n_qtiles * p.n_heads;
  p.work_per_xcd = (p.total_work + 7) / 8;
  constexpr size_t lds_bytes = 2 * kNBuf * kTileBytes;
  static bool attr_set = false;
  if (!attr_set) {
    SDVG_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(block_attn_bf16_pp_kernel<PRIO>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    attr_set = true;
  }
  hipLaunchKernelGGL(block_attn_bf16_pp_kernel<PRIO>, dim3(8 * p.work_per_xcd), dim3(512), lds_bytes,
                     s, p);
  SDVG_HIP_CHECK(hipGetLastError());
  return SDVG_OK;
}

template <int NW>
int launch_bf16(const AttnParams &p_in, hipStream_t s) {
  AttnParams p = p_in;
  constexpr int kBM = NW * 32;
  p.n_qtiles = (p.n_q + kBM - 1) / kBM;
  p.total_work = p.n_qtiles * p.n_heads;
  p.work_per_xcd = (p.total_work + 7) / 8;
  constexpr size_t lds_bytes = 2 * (kKTile + kVTile) * sizeof(uint16_t);
  static bool attr_set = false;  // raising the dynamic LDS limit is idempotent; races are benign
  if (!attr_set) {
    SDVG_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(block_attn_bf16_kernel<NW>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
    attr_set = true;
  }
  hipLaunchKernelGGL(block_attn_bf16_kernel<NW>, dim3(8 * p.work_per_xcd), dim3(NW * 64), lds_bytes,
                     s, p);
  SDVG_HIP_CHECK(hipGetLastError());
  return SDVG_OK;
}

}  // namespace

#ifdef SDVG_ATTN_TIMING
extern "C" int sdvg_debug_timing2(unsigned long long *host128) {
  return static_cast<int>(hipMemcpyFromSymbol(host128, HIP_SYMBOL(g_dbg2), sizeof(g_dbg2)));
}
extern "C" int sdvg_debug_timing(unsigned long long *host16) {
  return static_cast<int>(hipMemcpyFromSymbol(host16, HIP_SYMBOL(g_dbg), sizeof(g_dbg)));
}
#endif

extern "C" int sdvg_block_attn(const sdvg_attn_desc *desc, const void *q, const void *k_cache,
                               const void *v_cache, const void *k_blk, const void *v_blk,
                               int64_t cache_len, void *out, void *stream) {
  if (!desc || !q || !k_blk || !v_blk || !out) return SDVG_ERR_NULL;
  if (desc->head_dim != 128) return SDVG_ERR_UNSUPPORTED;
  if (desc->dtype != SDVG_BF16 && desc->dtype != SDVG_F32) return SDVG_ERR_UNSUPPORTED;
  if (desc->n_q < 1 || desc->n_blk < 1 || desc->n_heads < 1) return SDVG_ERR_SHAPE;
  if (cache_len < 0 || cache_len + desc->n_blk > INT32_MAX) return SDVG_ERR_RANGE;
  if (cache_len > 0 && (!k_cache || !v_cache)) return SDVG_ERR_NULL;
  if (!(desc->scale > 0.f) || !isfinite(desc->scale)) return SDVG_ERR_RANGE;
  const int64_t strides[] = {desc->q_token_stride, desc->q_head_stride, desc->o_token_stride,
                             desc->o_head_stride,  desc->blk_token_stride, desc->blk_head_stride};
  for (int64_t st : strides) {
    if (st < 128) return SDVG_ERR_SHAPE;
    if (st & 7) return SDVG_ERR_ALIGN;
  }
  if (cache_len > 0) {
    if (desc->kv_token_stride < 128 || desc->kv_head_stride < 128) return SDVG_ERR_SHAPE;
    if ((desc->kv_token_stride | desc->kv_head_stride) & 7) return SDVG_ERR_ALIGN;
    if (!sdvg::aligned16(k_cache) || !sdvg::aligned16(v_cache)) return SDVG_ERR_ALIGN;
  }
  if (!sdvg::aligned16(q) || !sdvg::aligned16(k_blk) || !sdvg::aligned16(v_blk) ||
      !sdvg::aligned16(out))
    return SDVG_ERR_ALIGN;
  if (desc->dtype == SDVG_F32) return SDVG_ERR_UNSUPPORTED;  // check path: not built yet

  AttnParams p{};
  p.q = static_cast<const uint16_t *>(q);
  p.k_cache = static_cast<const uint16_t *>(k_cache);
  p.v_cache = static_cast<const uint16_t *>(v_cache);
  p.k_blk = static_cast<const uint16_t *>(k_blk);
  p.v_blk = static_cast<const uint16_t *>(v_blk);
  p.out = static_cast<uint16_t *>(out);
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
  p.scale_log2e = desc->scale * 1.4426950408889634f;
  static const int variant = [] {
    const char *e = getenv("SDVG_ATTN_VARIANT");
    return e ? atoi(e) : 0;
  }();
  if (variant == 4) return launch_bf16<4>(p, static_cast<hipStream_t>(stream));
  if (variant == 20) return launch_bf16_pp2<0>(p, static_cast<hipStream_t>(stream));
  if (variant == 21) return launch_bf16_pp2<1>(p, static_cast<hipStream_t>(stream));
  if (variant == 22) return launch_bf16_pp2<2>(p, static_cast<hipStream_t>(stream));
  if (variant == 10) return launch_bf16_pp<0>(p, static_cast<hipStream_t>(stream));
  if (variant == 11) return launch_bf16_pp<1>(p, static_cast<hipStream_t>(stream));
  if (variant == 1) return launch_bf16<8>(p, static_cast<hipStream_t>(stream));
  return launch_bf16_pp2<1>(p, static_cast<hipStream_t>(stream));
}
