// fp32 check path of the block-causal attention (paper Sec. 1 / Sec. 4.1 "Models": one block's
// queries attend to the cached K/V of earlier blocks plus the block itself, no mask).
//
// Not a performance path: it exists so that the kernel skeleton -- transposed scores on the
// matrix cores, two-pointer cache/block concatenation, clamped tail loads, -inf masking,
// online softmax in the log2 domain, O^T accumulation, the epilogue layout -- can be checked
// against the fp64 oracle to 1e-4 without bf16 rounding in the way. Everything is fp32:
// v_mfma_f32_32x32x2_f32 for both products, fp32 probabilities, fp32 output.
//
// Workgroup = 4 wavefronts x 32 query rows of one head; K/V tiles of 32 keys staged through LDS
// (single buffer, two barriers per tile).
#include <math.h>

#include "block_attn_params.h"
#include "sdvg_common.h"

namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kBM = kWaves * 32;
constexpr int kBN = 32;        // keys per tile
constexpr int kStride = 132;   // LDS row stride in floats (128 + 4 pad)

__device__ __forceinline__ float other_half(float x) {
  // value of the lane 32 away
  return __shfl_xor(x, 32, 64);
}

__global__ __launch_bounds__(kThreads) void block_attn_f32_kernel(const sdvg::AttnParams p) {
  __shared__ __attribute__((aligned(16))) float lds_k[kBN * kStride];
  __shared__ __attribute__((aligned(16))) float lds_v[kBN * kStride];

  const int head = blockIdx.x / p.n_qtiles;
  const int qt = blockIdx.x - head * p.n_qtiles;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r32 = lane & 31, hh = lane >> 5;

  const float *q = static_cast<const float *>(p.items[0].q);
  const float *k_cache = static_cast<const float *>(p.items[0].k_cache);
  const float *v_cache = static_cast<const float *>(p.items[0].v_cache);
  const float *k_blk = static_cast<const float *>(p.items[0].k_blk);
  const float *v_blk = static_cast<const float *>(p.items[0].v_blk);
  float *out = static_cast<float *>(p.items[0].out);

  // Q fragments: B operand of S^T = K Q^T; lane holds Q[q_row][2*s + hh], s = 0..63
  const int q_row = qt * kBM + wave * 32 + r32;
  const int q_row_ld = q_row < p.n_q ? q_row : p.n_q - 1;
  float qf[64];
  {
    const float *qp = q + q_row_ld * p.q_ts + head * p.q_hs + hh;
#pragma unroll
    for (int s = 0; s < 64; ++s) qf[s] = qp[2 * s];
  }

  f32x16 o_acc[4];  // O^T: o_acc[db][i] = O[q_row][32*db + 8*(i/4) + 4*hh + i%4]
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o_acc[db][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int n_tiles = (p.n_k + kBN - 1) / kBN;
  for (int t = 0; t < n_tiles; ++t) {
    // ---- stage the tile: 32 keys x 32 float4 chunks for K and for V, 4 chunks per thread each
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int g = tid + u * kThreads;
      const int row = g >> 5, c = g & 31;
      int64_t j = static_cast<int64_t>(t) * kBN + row;
      j = j < p.n_k ? j : p.n_k - 1;  // never read past the last valid key; masked below
      const float *kp, *vp;
      if (j < p.cache_len) {
        const int64_t off = j * p.kv_ts + head * p.kv_hs + c * 4;
        kp = k_cache + off;
        vp = v_cache + off;
      } else {
        const int64_t off = (j - p.cache_len) * p.blk_ts + head * p.blk_hs + c * 4;
        kp = k_blk + off;
        vp = v_blk + off;
      }
      *reinterpret_cast<f32x4 *>(lds_k + row * kStride + c * 4) = *reinterpret_cast<const f32x4 *>(kp);
      *reinterpret_cast<f32x4 *>(lds_v + row * kStride + c * 4) = *reinterpret_cast<const f32x4 *>(vp);
    }
    __syncthreads();

    // ---- S^T = K Q^T (32 keys x 32 queries): lane holds key 8*(i/4) + 4*hh + i%4 of query r32
    f32x16 s_acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) s_acc[i] = 0.f;
#pragma unroll
    for (int s = 0; s < 64; ++s)
      s_acc = __builtin_amdgcn_mfma_f32_32x32x2f32(lds_k[r32 * kStride + 2 * s + hh], qf[s], s_acc, 0, 0, 0);

    if (t == n_tiles - 1) {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (t * kBN + 8 * (i >> 2) + 4 * hh + (i & 3) >= p.n_k) s_acc[i] = -INFINITY;
    }

    // ---- online softmax in the log2 domain (every tile holds at least one valid key)
    float mt = s_acc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mt = fmaxf(mt, s_acc[i]);
    mt = fmaxf(mt, other_half(mt)) * p.scale_log2e;
    const float m_new = fmaxf(m_run, mt);
    const float alpha = exp2f(m_run - m_new);  // 0 on the first tile
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      s_acc[i] = exp2f(s_acc[i] * p.scale_log2e - m_new);
      psum += s_acc[i];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o_acc[db][i] *= alpha;

    // ---- O^T += V^T P^T: register i of s_acc pairs key 8*(i/4)+i%4 (hh = 0) with the key 4 on
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = 8 * (i >> 2) + 4 * hh + (i & 3);
#pragma unroll
      for (int db = 0; db < 4; ++db)
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(lds_v[key * kStride + 32 * db + r32], s_acc[i],
                                                         o_acc[db], 0, 0, 0);
    }
    __syncthreads();
  }

  const float inv_l = 1.0f / (l_run + other_half(l_run));
  if (q_row < p.n_q) {
    float *op = out + q_row * p.o_ts + head * p.o_hs + 4 * hh;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 o4 = {o_acc[db][4 * g] * inv_l, o_acc[db][4 * g + 1] * inv_l,
                          o_acc[db][4 * g + 2] * inv_l, o_acc[db][4 * g + 3] * inv_l};
        *reinterpret_cast<f32x4 *>(op + 32 * db + 8 * g) = o4;
      }
  }
}

}  // namespace

int sdvg::launch_block_attn_f32(const sdvg::AttnParams &p_in, hipStream_t s) {
  sdvg::AttnParams p = p_in;
  p.n_qtiles = (p.n_q + kBM - 1) / kBM;
  hipLaunchKernelGGL(block_attn_f32_kernel, dim3(p.n_qtiles * p.n_heads), dim3(kThreads), 0, s, p);
  SDVG_HIP_CHECK(hipGetLastError());
  return SDVG_OK;
}
