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
  return launch_bf16<8>(p, static_cast<hipStream_t>(stream));
}
