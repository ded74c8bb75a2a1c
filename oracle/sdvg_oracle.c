/*
 * sdvg_oracle.c -- slow, plain CPU reference for the SDVG attention / KV-cache / routing path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it. It shares no code with the GPU library.
 *
 * What it computes (paper sections cited per function):
 *   - block attention: softmax(q K^T * scale) V with K, V = concat(cache[0:c], block) along
 *     tokens, no mask (one block's queries see the whole cache and the whole block).
 *     Paper Sec. 1 (shared KV cache) and Sec. 4.1 "Models" (causal attention backbone with
 *     KV caching); the mathematical statement is the textbook softmax attention.
 *   - KV commit / rollback: Sec. 3 "Inference flow" (accepted draft is committed to the
 *     target's KV cache; on reject the cache must look as if the draft was never there).
 *   - worst-frame routing: Sec. 3 Eq. (1) (min over frames), the accept rule q_b >= tau of
 *     "Inference flow", and "Force-reject the first block"; mode 1 is the average-frame variant
 *     of the ablation (Sec. 4.3 "Min-frame vs. average-frame scoring").
 *   - snapshot / restore of an opaque buffer: Sec. 3 "Inference flow" (VAE decode cache cloned
 *     before scoring, restored on rejection): a byte copy.
 *   - rotary position embedding of q / k rows: Sec. 4.1 "Models" (KV caching "via RoPE positional
 *     embeddings"; the paper prints no formula -- the reading taken is at the function).
 *
 * Everything is fp64, two-pass, materialised-row: deliberately NOT tiled / online.
 * Element types: 0 = bfloat16 bit patterns (uint16), 1 = float32. Both widen exactly to fp64.
 * All strides are in elements. Index order everywhere: (layer, token, head, dim).
 *
 * Every function here has an independent pin in tests/test_oracle_*.py; none is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_BF16 0
#define ORACLE_F32 1

static double widen(const void *base, int64_t idx, int dtype) {
  if (dtype == ORACLE_BF16) {
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16; /* bf16 = top half of f32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
  }
  return (double)((const float *)base)[idx];
}

/*
 * Attention for a list of query rows (rows == NULL means rows 0..n_rows-1).
 * out is dense fp64 [n_rows][n_heads][head_dim]. weights_out (nullable) receives the
 * normalised softmax weights, dense [n_rows][n_heads][cache_len + n_blk], for invariant tests.
 * Returns 0, or -1 on allocation failure / bad arguments.
 */
int sdvg_oracle_block_attn(const void *q, const void *k_cache, const void *v_cache,
                           const void *k_blk, const void *v_blk, int dtype,
                           int64_t n_blk, int64_t n_heads, int64_t head_dim, int64_t cache_len,
                           int64_t q_token_stride, int64_t q_head_stride,
                           int64_t kv_token_stride, int64_t kv_head_stride,
                           int64_t blk_token_stride, int64_t blk_head_stride,
                           double scale, const int64_t *rows, int64_t n_rows,
                           double *out, double *weights_out) {
  const int64_t n_k = cache_len + n_blk;
  if (n_k <= 0 || n_rows < 0 || head_dim <= 0 || n_heads <= 0) return -1;
  int failed = 0;
#pragma omp parallel
  {
    double *s = (double *)malloc((size_t)n_k * sizeof(double));
    if (!s) {
#pragma omp atomic write
      failed = 1;
    }
#pragma omp for collapse(2) schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
      for (int64_t h = 0; h < n_heads; ++h) {
        if (!s) continue;
        const int64_t i = rows ? rows[r] : r;
        const int64_t qoff = i * q_token_stride + h * q_head_stride;
        /* logits over cache tokens, then block tokens */
        for (int64_t j = 0; j < n_k; ++j) {
          const void *kb = (j < cache_len) ? k_cache : k_blk;
          const int64_t koff = (j < cache_len)
                                   ? j * kv_token_stride + h * kv_head_stride
                                   : (j - cache_len) * blk_token_stride + h * blk_head_stride;
          double dot = 0.0;
          for (int64_t t = 0; t < head_dim; ++t)
            dot += widen(q, qoff + t, dtype) * widen(kb, koff + t, dtype);
          s[j] = dot * scale;
        }
        double m = s[0];
        for (int64_t j = 1; j < n_k; ++j)
          if (s[j] > m) m = s[j];
        double z = 0.0;
        for (int64_t j = 0; j < n_k; ++j) {
          s[j] = exp(s[j] - m);
          z += s[j];
        }
        double *o = out + (r * n_heads + h) * head_dim;
        for (int64_t t = 0; t < head_dim; ++t) o[t] = 0.0;
        for (int64_t j = 0; j < n_k; ++j) {
          const void *vb = (j < cache_len) ? v_cache : v_blk;
          const int64_t voff = (j < cache_len)
                                   ? j * kv_token_stride + h * kv_head_stride
                                   : (j - cache_len) * blk_token_stride + h * blk_head_stride;
          for (int64_t t = 0; t < head_dim; ++t) o[t] += s[j] * widen(vb, voff + t, dtype);
        }
        for (int64_t t = 0; t < head_dim; ++t) o[t] /= z;
        if (weights_out) {
          double *w = weights_out + (r * n_heads + h) * n_k;
          for (int64_t j = 0; j < n_k; ++j) w[j] = s[j] / z;
        }
      }
    }
    free(s);
  }
  return failed ? -1 : 0;
}

/*
 * Host mirror of the KV cache: two arrays of 16-bit words, logical
 * [n_layers][capacity_tokens][n_heads][head_dim], dense. cache_len is passed by pointer and
 * updated like the real cache's host field.
 *
 * Commit (Sec. 3 "Inference flow", accept branch; also the unconditional drafter-cache update):
 * copy block [n_layers][T][n_heads][head_dim] into tokens [slot*T, (slot+1)*T) of every layer.
 * Append-only: slot*T must equal *cache_len. Returns 0, or -3 if the slot is out of range.
 */
int sdvg_oracle_kv_commit(uint16_t *cache_k, uint16_t *cache_v, int64_t n_layers,
                          int64_t capacity_tokens, int64_t n_heads, int64_t head_dim,
                          int64_t block_tokens, int64_t *cache_len, const uint16_t *k_blk,
                          const uint16_t *v_blk, int64_t slot) {
  if (slot < 0 || slot * block_tokens != *cache_len ||
      (slot + 1) * block_tokens > capacity_tokens)
    return -3;
  for (int64_t l = 0; l < n_layers; ++l)
    for (int64_t t = 0; t < block_tokens; ++t)
      for (int64_t h = 0; h < n_heads; ++h)
        for (int64_t x = 0; x < head_dim; ++x) {
          const int64_t src = ((l * block_tokens + t) * n_heads + h) * head_dim + x;
          const int64_t dst =
              ((l * capacity_tokens + slot * block_tokens + t) * n_heads + h) * head_dim + x;
          cache_k[dst] = k_blk[src];
          cache_v[dst] = v_blk[src];
        }
  *cache_len = (slot + 1) * block_tokens;
  return 0;
}

/*
 * Rollback (Sec. 3 "Inference flow", reject branch): truncate to new_len and zero the words
 * of tokens [new_len, old_len) in every layer, so no trace of the rejected draft remains.
 * Returns 0, or -3 if new_len is outside [0, *cache_len].
 */
int sdvg_oracle_kv_rollback(uint16_t *cache_k, uint16_t *cache_v, int64_t n_layers,
                            int64_t capacity_tokens, int64_t n_heads, int64_t head_dim,
                            int64_t *cache_len, int64_t new_len) {
  if (new_len < 0 || new_len > *cache_len) return -3;
  for (int64_t l = 0; l < n_layers; ++l)
    for (int64_t t = new_len; t < *cache_len; ++t)
      for (int64_t h = 0; h < n_heads; ++h)
        for (int64_t x = 0; x < head_dim; ++x) {
          const int64_t dst = ((l * capacity_tokens + t) * n_heads + h) * head_dim + x;
          cache_k[dst] = 0;
          cache_v[dst] = 0;
        }
  *cache_len = new_len;
  return 0;
}

/*
 * Worst-frame routing. Sec. 3 Eq. (1): q_b = min_i score_i; accept iff q_b >= tau
 * ("Inference flow"); block 0 is always rejected ("Force-reject the first block") but its
 * true q_b is still reported. mode 1 is the ablation's mean aggregation (Sec. 4.3), summed
 * sequentially in fp64 and rounded once to fp32.
 * Readings where the paper is silent: any NaN score -> reject with q_b = quiet NaN 0x7FC00000;
 * among equal zeros the negative one is the minimum, so q_b is unique under any scan order.
 * Returns 1 accept, 0 reject.
 */
int sdvg_oracle_route(const float *scores, int64_t n_frames, float tau, int64_t block_idx,
                      int mode, float *q_b_out) {
  float qb;
  int has_nan = 0;
  for (int64_t i = 0; i < n_frames; ++i)
    if (isnan(scores[i])) has_nan = 1;
  if (has_nan) {
    const uint32_t qnan = 0x7FC00000u;
    memcpy(&qb, &qnan, sizeof qb);
    if (q_b_out) *q_b_out = qb;
    return 0;
  }
  if (mode == 1) {
    double acc = 0.0;
    for (int64_t i = 0; i < n_frames; ++i) acc += (double)scores[i];
    qb = (float)(acc / (double)n_frames);
    if (isnan(qb)) { /* +inf and -inf among the scores: same canonical NaN as a NaN score */
      const uint32_t qnan = 0x7FC00000u;
      memcpy(&qb, &qnan, sizeof qb);
      if (q_b_out) *q_b_out = qb;
      return 0;
    }
  } else {
    qb = scores[0];
    for (int64_t i = 1; i < n_frames; ++i) {
      const float s = scores[i];
      if (s < qb || (s == qb && signbit(s) && !signbit(qb))) qb = s;
    }
  }
  if (q_b_out) *q_b_out = qb;
  return (block_idx != 0 && qb >= tau) ? 1 : 0;
}

/*
 * Snapshot / restore of an opaque buffer (paper Sec. 3 "Inference flow": the VAE decode cache is
 * cloned before draft scoring and restored on rejection): dst[i] = src[i], byte by byte.
 */
int sdvg_oracle_buffer_copy(uint8_t *dst, const uint8_t *src, int64_t n_bytes) {
  if (n_bytes < 0) return -2;
  for (int64_t i = 0; i < n_bytes; ++i) dst[i] = src[i];
  return 0;
}

/*
 * Rotary position embedding (paper Sec. 4.1 "Models" names RoPE and nothing more). Reading taken:
 * the standard rotation of consecutive pairs -- element 2i and 2i+1 of a head's vector are the
 * real and imaginary part of a complex number that is multiplied by exp(i * angle) -- with the
 * angle of (token, pair) supplied by the caller as tables cos[token][head_dim/2] and
 * sin[token][head_dim/2] (fp32), so that any position scheme (1-D, or the 3-D frame/row/column
 * scheme of video transformers) is the caller's choice and not part of this function.
 * Input and output are bf16 bit patterns, dense [n_tokens][n_heads][head_dim]. The arithmetic is
 * the kernel's precision, fp32, in a fixed order, because the result is rounded to bf16 and both
 * sides must take that rounding decision from the same fp32 value:
 *     re' = fma(re, cos, -(im * sin)),   im' = fma(re, sin, im * cos),
 * each product and each fma rounded once to fp32, then round-to-nearest-even to bf16.
 * Returns 0, or -2 on a bad shape.
 */
static uint16_t bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, sizeof u);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x0040u); /* NaN */
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

int sdvg_oracle_rope(const uint16_t *x, const float *cos_t, const float *sin_t, uint16_t *out,
                     int64_t n_tokens, int64_t n_heads, int64_t head_dim) {
  if (n_tokens < 0 || n_heads <= 0 || head_dim <= 0 || (head_dim & 1)) return -2;
  const int64_t half = head_dim / 2;
  for (int64_t t = 0; t < n_tokens; ++t)
    for (int64_t h = 0; h < n_heads; ++h)
      for (int64_t i = 0; i < half; ++i) {
        const int64_t e = (t * n_heads + h) * head_dim + 2 * i;
        const float re = (float)widen(x, e, ORACLE_BF16), im = (float)widen(x, e + 1, ORACLE_BF16);
        const float c = cos_t[t * half + i], sn = sin_t[t * half + i];
        const volatile float im_sin = im * sn; /* volatile: each product is rounded to fp32 on its own */
        const volatile float im_cos = im * c;
        out[e] = bf16_rne(fmaf(re, c, -im_sin));
        out[e + 1] = bf16_rne(fmaf(re, sn, im_cos));
      }
  return 0;
}

/* Threads the attention loop above will use (reported beside the timed baseline). */
int sdvg_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
