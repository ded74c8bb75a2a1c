// Rotary position embedding of q / k rows, alone and fused into the KV commit.
// Paper Sec. 4.1 "Models": the attention backbone caches K/V "via RoPE positional embeddings"; no
// formula is printed. Reading taken: consecutive elements (2i, 2i+1) of a head's vector are the
// real and imaginary part of a complex number that is multiplied by exp(i * angle), the angle of
// (token, pair) being supplied by the caller as fp32 tables cos / sin [token][64] -- so the position
// scheme (1-D, or the 3-D frame / row / column scheme of video transformers) stays the caller's.
// Arithmetic: fp32 in a fixed order (each product and each fma rounded once), result rounded to
// bf16 (RNE):  re' = fma(re, cos, -(im * sin)),  im' = fma(re, sin, im * cos).
//
// Why K is rotated on its way INTO the cache and not "on load" in the attention kernel: K tiles
// go from HBM to LDS without passing through registers, and every one of a head's 19 workgroups
// would have to rotate every tile again. Rotating once, in the bandwidth-bound copy that commits
// the block, costs nothing; q and the current block's K are rotated by the plain kernel (one
// pass over 48 MB in and out per tensor and layer at the target shape, 17 us against 2.4 ms of attention).
#include "sdvg_common.h"

namespace {

typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int kThreads = 256;

// Rotates the four pairs held in one 16-byte chunk (8 bf16) by the angles (c[i], s[i]).
__device__ __forceinline__ u32x4 rotate_chunk(u32x4 x, f32x4 c, f32x4 s) {
  u32x4 y;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float re = __uint_as_float(x[i] << 16), im = __uint_as_float(x[i] & 0xffff0000u);
    const float im_sin = __fmul_rn(im, s[i]), im_cos = __fmul_rn(im, c[i]);
    const f32x2 r = {__fmaf_rn(re, c[i], -im_sin), __fmaf_rn(re, s[i], im_cos)};
    const bf16x2 b = __builtin_convertvector(r, bf16x2);
    unsigned int packed;
    __builtin_memcpy(&packed, &b, 4);
    y[i] = packed;
  }
  return y;
}

// One 16-byte chunk per thread: chunk g = (token, head, chunk-in-row).
__global__ __launch_bounds__(kThreads) void rope_kernel(const uint16_t *__restrict__ x, const float *__restrict__ cos_t,
                                                        const float *__restrict__ sin_t, uint16_t *out,
                                                        int64_t n_chunks, int n_heads, int64_t x_ts, int64_t x_hs,
                                                        int64_t o_ts, int64_t o_hs) {
  const int64_t g = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (g >= n_chunks) return;
  const int ch = static_cast<int>(g & 15);
  const int64_t row = g >> 4;
  const int64_t tok = row / n_heads;
  const int head = static_cast<int>(row - tok * n_heads);
  const u32x4 v = *reinterpret_cast<const u32x4 *>(x + tok * x_ts + head * x_hs + ch * 8);
  const f32x4 c = *reinterpret_cast<const f32x4 *>(cos_t + tok * 64 + ch * 4);
  const f32x4 s = *reinterpret_cast<const f32x4 *>(sin_t + tok * 64 + ch * 4);
  *reinterpret_cast<u32x4 *>(out + tok * o_ts + head * o_hs + ch * 8) = rotate_chunk(v, c, s);
}

// Commit with the rotation of K fused in: grid.y = layer, grid.z = 0 (K, rotated) / 1 (V, copied).
// Source dense [L][T][H][128]; destination addressed with the cache's strides.
__global__ __launch_bounds__(kThreads) void kv_commit_rope_kernel(
    const uint16_t *__restrict__ k_src, const uint16_t *__restrict__ v_src, uint16_t *__restrict__ k_dst,
    uint16_t *__restrict__ v_dst, const float *__restrict__ cos_t, const float *__restrict__ sin_t,
    int64_t chunks_per_layer, int n_heads, int64_t layer_stride, int64_t token_stride, int64_t head_stride,
    int64_t first_token) {
  const int64_t g = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (g >= chunks_per_layer) return;
  const bool is_v = blockIdx.z != 0;
  const int ch = static_cast<int>(g & 15);
  const int64_t row = g >> 4;
  const int64_t tok = row / n_heads;
  const int head = static_cast<int>(row - tok * n_heads);
  const uint16_t *src = (is_v ? v_src : k_src) + (blockIdx.y * chunks_per_layer + g) * 8;
  uint16_t *dst = (is_v ? v_dst : k_dst) + blockIdx.y * layer_stride + (first_token + tok) * token_stride +
                  head * head_stride + ch * 8;
  u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
  if (!is_v) {
    const f32x4 c = *reinterpret_cast<const f32x4 *>(cos_t + tok * 64 + ch * 4);
    const f32x4 s = *reinterpret_cast<const f32x4 *>(sin_t + tok * 64 + ch * 4);
    v = rotate_chunk(v, c, s);
  }
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(dst));
}

bool stride_ok(int64_t st) { return st >= 128 && (st & 7) == 0; }

}  // namespace

extern "C" int sdvg_rope(const void *x, const float *cos_table, const float *sin_table, void *out,
                         int64_t n_tokens, int32_t n_heads, int32_t head_dim, int64_t x_token_stride,
                         int64_t x_head_stride, int64_t out_token_stride, int64_t out_head_stride, void *stream) {
  if (n_tokens < 0 || n_heads < 1) return SDVG_ERR_SHAPE;
  if (head_dim != 128) return SDVG_ERR_UNSUPPORTED;
  if (n_tokens == 0) return SDVG_OK;
  if (!x || !cos_table || !sin_table || !out) return SDVG_ERR_NULL;
  if (!stride_ok(x_token_stride) || !stride_ok(x_head_stride) || !stride_ok(out_token_stride) ||
      !stride_ok(out_head_stride))
    return (x_token_stride < 128 || x_head_stride < 128 || out_token_stride < 128 || out_head_stride < 128)
               ? SDVG_ERR_SHAPE
               : SDVG_ERR_ALIGN;
  if (!sdvg::aligned16(x) || !sdvg::aligned16(out) || !sdvg::aligned16(cos_table) || !sdvg::aligned16(sin_table))
    return SDVG_ERR_ALIGN;
  const int64_t n_chunks = n_tokens * n_heads * 16;
  const int64_t blocks = (n_chunks + kThreads - 1) / kThreads;
  if (blocks > 0x7FFFFFFF) return SDVG_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(rope_kernel, dim3(static_cast<unsigned>(blocks)), dim3(kThreads), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint16_t *>(x), cos_table, sin_table,
                     static_cast<uint16_t *>(out), n_chunks, n_heads, x_token_stride, x_head_stride,
                     out_token_stride, out_head_stride);
  SDVG_HIP_CHECK(hipGetLastError());
  return SDVG_OK;
}

extern "C" int sdvg_kv_commit_rope(sdvg_kv_cache *cache, const void *k_blk, const void *v_blk, int32_t slot,
                                   const float *cos_table, const float *sin_table, void *stream) {
  if (!cos_table || !sin_table) return SDVG_ERR_NULL;
  if (!sdvg::aligned16(cos_table) || !sdvg::aligned16(sin_table)) return SDVG_ERR_ALIGN;
  // the same checks as the plain commit (descriptor, slot, alignment, aliasing), without a launch
  int st = sdvg::check_commit_args(cache, k_blk, v_blk, slot);
  if (st != SDVG_OK) return st;
  const int64_t T = cache->block_tokens;
  const int64_t chunks_per_layer = T * cache->n_heads * 16;
  const dim3 grid(static_cast<unsigned>((chunks_per_layer + kThreads - 1) / kThreads), cache->n_layers, 2);
  hipLaunchKernelGGL(kv_commit_rope_kernel, grid, dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint16_t *>(k_blk), static_cast<const uint16_t *>(v_blk),
                     static_cast<uint16_t *>(cache->k), static_cast<uint16_t *>(cache->v), cos_table, sin_table,
                     chunks_per_layer, cache->n_heads, cache->layer_stride, cache->token_stride, cache->head_stride,
                     static_cast<int64_t>(slot) * T);
  SDVG_HIP_CHECK(hipGetLastError());
  cache->cache_len = (slot + 1) * T;
  return SDVG_OK;
}
