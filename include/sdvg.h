/*
 * sdvg.h -- C ABI of libsdvg: block-causal attention over a KV cache, KV-cache commit and
 * rollback, and worst-frame routing, for speculative decoding of autoregressive video
 * generation (SDVG) on AMD MI355X (gfx950).
 *
 * Conventions shared by every call
 *   - Pointers named "device" are HIP device pointers owned by the caller; the library never
 *     frees or reallocates them. Pointers named "host" are ordinary host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Every call returns an int: >= 0 on success, a negative sdvg_status on error. Arguments
 *     are validated on the host before anything is launched; on error nothing is launched
 *     and no state (device memory, descriptor fields) is changed. No call throws or aborts.
 *   - Strides are in elements of the tensor's type; the innermost (dim) stride is always 1.
 *   - Logical index order is (layer, token, head, dim). head_dim must be 128.
 *   - bf16 tensors are raw bfloat16 bit patterns (2 bytes per element).
 */
#ifndef SDVG_H
#define SDVG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SDVG_OK = 0,
  SDVG_ERR_NULL = -1,        /* a required pointer is NULL */
  SDVG_ERR_SHAPE = -2,       /* a size is non-positive or inconsistent */
  SDVG_ERR_RANGE = -3,       /* slot / length / threshold outside its valid range */
  SDVG_ERR_ALIGN = -4,       /* pointer not 16-byte aligned, or stride not a multiple of 8 */
  SDVG_ERR_UNSUPPORTED = -5, /* head_dim != 128, unknown dtype, stride >= 2^30 elements */
  SDVG_ERR_DEVICE = -6       /* a HIP runtime call failed (see sdvg_last_device_error) */
} sdvg_status;

enum { SDVG_BF16 = 0, SDVG_F32 = 1 };

/* Key-split policy of sdvg_block_attn_batch (see there). */
enum { SDVG_SPLIT_NEVER = 0, SDVG_SPLIT_AUTO = 1, SDVG_SPLIT_ALWAYS = 2 };

/*
 * Describes the caller-owned KV cache of one model: two device arrays k and v of bf16,
 * logical [n_layers][capacity_tokens][n_heads][head_dim]. cache_len is a HOST field: the
 * number of valid tokens (the same in every layer); commit and rollback update it at enqueue
 * time, so later calls on the same stream see a consistent length.
 */
typedef struct {
  void *k, *v;              /* device */
  int32_t n_layers, n_heads, head_dim;
  int32_t block_tokens;     /* T: tokens per video block (3 latent frames) */
  int64_t capacity_tokens;  /* tokens allocated per layer */
  int64_t cache_len;        /* valid tokens, 0 <= cache_len <= capacity_tokens */
  int64_t layer_stride, token_stride, head_stride; /* elements */
} sdvg_kv_cache;

/* Shapes and strides of one attention call (one layer, one denoising step). */
typedef struct {
  int32_t n_q;      /* query tokens of the current block */
  int32_t n_blk;    /* key/value tokens of the current block (normally == n_q) */
  int32_t n_heads;
  int32_t head_dim; /* must be 128 */
  int64_t q_token_stride, q_head_stride;     /* q */
  int64_t o_token_stride, o_head_stride;     /* out */
  int64_t kv_token_stride, kv_head_stride;   /* k_cache, v_cache (one layer) */
  int64_t blk_token_stride, blk_head_stride; /* k_blk, v_blk */
  float scale;      /* softmax scale; 0 selects 1/sqrt(head_dim), the paper's models' value */
  int32_t dtype;    /* SDVG_BF16: all tensors bf16. SDVG_F32: all tensors fp32 (check path) */
} sdvg_attn_desc;

/*
 * Block-causal attention of one video block over the KV cache (paper Sec. 1: blocks are
 * generated against a shared KV cache; Sec. 4.1 "Models": causal attention backbone with KV
 * caching). For every head h and query row i:
 *     out[i,h,:] = sum_j p_ij V[j,h,:],   p_i = softmax_j(scale * q[i,h,:] . K[j,h,:]),
 * where K, V are the cache's first cache_len tokens followed by the block's n_blk tokens.
 * No mask: a block's queries see the whole cache and the whole block.
 *   desc      host. Shapes, strides, scale, dtype.
 *   q         device [n_q][n_heads][128]; k_blk, v_blk device [n_blk][n_heads][128].
 *   k_cache, v_cache  device, ONE layer's base pointers, at least cache_len tokens; may be
 *             NULL when cache_len == 0. Tokens at or past cache_len are never read.
 *   out       device [n_q][n_heads][128], same dtype as the inputs; every element is written.
 *   Arithmetic (bf16): products on the matrix cores with fp32 accumulation, fp32 softmax
 *   statistics, probabilities rounded to bf16 before the PV product (the row sum is taken over
 *   the rounded values), bf16 output (RNE). SDVG_F32 is a slow all-fp32 check path: a separate,
 *   simple kernel that validates the mathematics (softmax over the concatenation) to 1e-4; it
 *   shares no tiling or copy logic with the bf16 kernel and says nothing about that kernel's
 *   indexing.
 *   scale must be finite and >= 0 (0 = 1/sqrt(head_dim)), else SDVG_ERR_RANGE. Inputs are
 *   assumed finite.
 * Asynchronous: enqueued on `stream`; returns SDVG_OK or a negative status. The call only
 * launches a kernel, so it may be recorded into a HIP graph -- but the first SDVG_BF16 call on
 * a device also raises that kernel's dynamic-LDS limit (once per device, thread-safe), which
 * is not a capturable operation: make one eager call on the device before capturing.
 */
int sdvg_block_attn(const sdvg_attn_desc *desc, const void *q, const void *k_cache,
                    const void *v_cache, const void *k_blk, const void *v_blk,
                    int64_t cache_len, void *out, void *stream);

/*
 * Attention with the commit fused in (paper Sec. 3 "Inference flow": the block the target keeps
 * -- an accepted draft, or the target's own regeneration -- updates its KV cache): sdvg_block_attn
 * for one layer (bf16 only), and in the same launch the block's K and V rows are copied into
 * tokens [cache_len, cache_len + n_blk) of k_cache / v_cache (this layer's base pointers, which
 * must have room for them), addressed with the descriptor's kv strides. Meant for the LAST
 * denoising step of a block: the copy runs on compute units the attention leaves idle, so the
 * block's commit costs no extra pass over memory. The attention result is bit-identical to
 * sdvg_block_attn's; the copied rows are bit-exact. k_blk / v_blk must not overlap the
 * destination rows (SDVG_ERR_RANGE). The cache length is the caller's to advance: after the
 * call has been made for every layer, sdvg_kv_commit_mark(cache, slot) moves the descriptor's
 * cache_len to (slot + 1) * T under the same append-only rule as sdvg_kv_commit, without
 * touching device memory. Asynchronous on `stream`.
 */
int sdvg_block_attn_commit(const sdvg_attn_desc *desc, const void *q, void *k_cache, void *v_cache,
                           const void *k_blk, const void *v_blk, int64_t cache_len, void *out,
                           void *stream);
int sdvg_kv_commit_mark(sdvg_kv_cache *cache, int32_t slot);

/*
 * The same attention for up to 8 independent (q, cache, block, out) sets in ONE launch -- e.g. the
 * conditional and the unconditional pass of classifier-free guidance (paper Sec. 4.1 "Models":
 * guidance scale 3.0), which share shapes and cache length but have their own tensors. Result
 * item by item as n_items calls of sdvg_block_attn; one launch fills the chip better and halves
 * the launch count.
 *   n_items   1 .. 8. q, k_cache, v_cache, k_blk, v_blk, out: HOST arrays of n_items device
 *             pointers (k_cache / v_cache and their entries may be NULL when cache_len == 0).
 *             All items share desc (shapes, strides, scale, dtype) and cache_len.
 *   workspace device, nullable, 16-byte aligned, workspace_bytes long; split_mode one of
 *             SDVG_SPLIT_*. Without a workspace (or with SDVG_SPLIT_NEVER) every query tile of
 *             256 rows is one workgroup. With a workspace of at least
 *             sdvg_block_attn_workspace_bytes(desc, n_items, cache_len, split_mode) bytes the
 *             library may deal the (query tile, key tile) pairs out evenly over whole rounds of
 *             workgroups instead, so that a launch with few query tiles still fills the chip,
 *             and merge the partial results of the query tiles that were cut in a second small
 *             kernel on the same stream. SDVG_SPLIT_AUTO does so when at least 60 % of the last
 *             round of workgroups would idle (very few heads or short blocks); SDVG_SPLIT_ALWAYS
 *             whenever the query tiles do not fill whole rounds. For the paper's own shapes the
 *             split does not pay (a 12-head drafter layer has 228 query tiles for 256 compute
 *             units; the split costs more than the 11 % it could win) and AUTO leaves them alone.
 *             Same softmax and same error bounds; not bit-identical to the unsplit result (P is
 *             rounded to bf16 against each piece's own running maximum). A workspace that is
 *             too small is ignored (plain launch). The workspace is scratch: contents are
 *             undefined afterwards; concurrent calls need their own.
 * Errors as sdvg_block_attn, plus SDVG_ERR_SHAPE for n_items outside 1 .. 8 or a negative
 * workspace_bytes and SDVG_ERR_UNSUPPORTED for an unknown split_mode. Asynchronous on `stream`.
 */
int sdvg_block_attn_batch(const sdvg_attn_desc *desc, int32_t n_items, const void *const *q,
                          const void *const *k_cache, const void *const *v_cache,
                          const void *const *k_blk, const void *const *v_blk, int64_t cache_len,
                          void *const *out, void *workspace, int64_t workspace_bytes,
                          int32_t split_mode, void *stream);

/*
 * sdvg_block_attn_batch for callers that cannot allocate device memory or provide a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same
 * arguments, results and errors, but the partial results of a key split go to a fixed 64 MiB
 * array inside the library's device image (sdvg_block_attn_static_workspace_limit() bytes,
 * held by every GPU the library runs on until the process ends) instead of caller memory.
 * The call allocates nothing and frees nothing. A shape whose split needs more than the array
 * holds returns SDVG_ERR_RANGE (nothing is launched); sdvg_block_attn_workspace_bytes tells the
 * need beforehand, and SDVG_SPLIT_NEVER needs none. Every call on a GPU uses that GPU's one
 * array: calls that overlap in time on one GPU (different streams or threads) race -- serialise
 * them, or use sdvg_block_attn_batch with workspaces of their own. Nothing in the array has to
 * be cleared between calls: each call writes every partial result it later reads.
 */
int sdvg_block_attn_batch_static(const sdvg_attn_desc *desc, int32_t n_items, const void *const *q,
                                 const void *const *k_cache, const void *const *v_cache,
                                 const void *const *k_blk, const void *const *v_blk, int64_t cache_len,
                                 void *const *out, int32_t split_mode, void *stream);
int64_t sdvg_block_attn_static_workspace_limit(void);

/*
 * Bytes of workspace with which sdvg_block_attn_batch would split keys for this shape and
 * split_mode on the current device; 0 if it would not split (then no workspace is needed).
 * Negative sdvg_status on a bad descriptor.
 */
int64_t sdvg_block_attn_workspace_bytes(const sdvg_attn_desc *desc, int32_t n_items, int64_t cache_len,
                                        int32_t split_mode);

/*
 * KV commit (paper Sec. 3 "Inference flow": an accepted draft block is committed to the
 * target's KV cache; a regenerated block updates it; the drafter's own cache is updated
 * unconditionally). Copies k_blk, v_blk -- device, dense [n_layers][T][n_heads][128] bf16 --
 * into tokens [slot*T, (slot+1)*T) of every layer, then sets cache->cache_len = (slot+1)*T.
 * Append-only: requires slot*T == cache->cache_len and (slot+1)*T <= capacity_tokens, else
 * SDVG_ERR_RANGE. k_blk / v_blk must not overlap the destination slot of any layer
 * (SDVG_ERR_RANGE). The descriptor's strides must keep rows and layers apart: the larger of
 * token_stride and head_stride steps over everything the smaller one spans, and layer_stride
 * over a whole layer (SDVG_ERR_SHAPE otherwise; the same check guards sdvg_kv_rollback).
 * One launch covers all layers. Asynchronous on `stream`.
 */
int sdvg_kv_commit(sdvg_kv_cache *cache, const void *k_blk, const void *v_blk, int32_t slot,
                   void *stream);

/*
 * Rotary position embedding of q / k rows (paper Sec. 4.1 "Models": KV caching "via RoPE positional
 * embeddings"; no formula is printed). Reading taken: elements 2i and 2i+1 of every head's vector
 * are the real and imaginary part of a complex number that is multiplied by exp(i * angle); the
 * angle of (token, pair i) is given by the caller as tables, so the position scheme is the
 * caller's. fp32 arithmetic in a fixed order, bf16 result (RNE):
 *     re' = fma(re, cos, -(im * sin)),   im' = fma(re, sin, im * cos).
 *   x, out     device bf16 [n_tokens][n_heads][128] with the given token / head strides
 *              (elements; multiples of 8, >= 128); out may be x itself (in place), otherwise the
 *              two must not overlap.
 *   cos_table, sin_table  device fp32, dense [n_tokens][64], 16-byte aligned.
 * head_dim must be 128. n_tokens == 0 is a no-op. Asynchronous on `stream`.
 */
int sdvg_rope(const void *x, const float *cos_table, const float *sin_table, void *out,
              int64_t n_tokens, int32_t n_heads, int32_t head_dim, int64_t x_token_stride,
              int64_t x_head_stride, int64_t out_token_stride, int64_t out_head_stride, void *stream);

/*
 * sdvg_kv_commit with the rotation of K fused into the copy: k_blk holds the block's keys BEFORE
 * the rotary embedding; they are rotated (as sdvg_rope, tables [T][64] shared by all layers) on
 * their way into the cache, v_blk is copied as it is. One pass over the block instead of two,
 * and the cache holds rotated keys, which is what sdvg_block_attn expects to find there. (Keys
 * are not rotated "on load" inside the attention kernel: its K tiles go from HBM to LDS without
 * passing registers, and each of a head's workgroups would rotate every tile again.)
 * Arguments, rules and errors otherwise as sdvg_kv_commit.
 */
int sdvg_kv_commit_rope(sdvg_kv_cache *cache, const void *k_blk, const void *v_blk, int32_t slot,
                        const float *cos_table, const float *sin_table, void *stream);

/*
 * KV rollback (paper Sec. 3 "Inference flow", reject branch: the target regenerates the block
 * as if the draft had never been in its cache). Sets cache->cache_len = new_len and zero-fills
 * tokens [new_len, old cache_len) of k and v in every layer, so no rejected data survives.
 * Requires 0 <= new_len <= cache->cache_len, else SDVG_ERR_RANGE; equal lengths is a no-op.
 * Asynchronous on `stream`.
 */
int sdvg_kv_rollback(sdvg_kv_cache *cache, int64_t new_len, void *stream);

/*
 * Snapshot / restore of an opaque device buffer (paper Sec. 3 "Inference flow" and Sec. 4.1
 * "Hardware and implementation": the VAE decode cache is cloned before a draft is scored and
 * restored when the draft is rejected). One call copies n_bytes from src to dst; cloning is
 * (snapshot <- live), restoring is (live <- snapshot). The library knows nothing of the contents.
 *   dst, src  device, 16-byte aligned, caller-owned, must not overlap (SDVG_ERR_RANGE).
 *   n_bytes   >= 0; 0 is a no-op that touches nothing (pointers may then be NULL).
 * Bit-exact; bytes outside [dst, dst + n_bytes) are not written. Asynchronous on `stream`.
 */
int sdvg_buffer_snapshot(void *dst, const void *src, int64_t n_bytes, void *stream);

/*
 * Worst-frame routing (paper Sec. 3 Eq. (1): q_b = min over the block's F decoded frames of
 * the per-frame reward; "Inference flow": accept iff q_b >= tau; "Force-reject the first
 * block": block 0 is always rejected, whatever its score).
 *   frame_scores  device, n_frames fp32 rewards (n_frames >= 1).
 *   tau           threshold; NaN -> SDVG_ERR_RANGE.
 *   block_idx     >= 0.
 *   q_b_out       host, nullable: receives q_b (also for block 0).
 * Any NaN score -> reject with q_b = quiet NaN (bits 0x7FC00000). Of +0.0 and -0.0 the
 * negative zero is the smaller, so q_b is bit-exact under any reduction order.
 * Synchronises `stream` (the caller branches on the result, as the paper's loop does).
 * Returns 1 (accept), 0 (reject) or a negative status.
 */
int sdvg_worst_frame_route(const float *frame_scores, int32_t n_frames, float tau,
                           int32_t block_idx, float *q_b_out, void *stream);

/*
 * Batched, asynchronous form of the same rule for n_blocks blocks at once.
 *   frame_scores  device [n_blocks][n_frames] fp32, dense.
 *   block_idx     device, n_blocks int32 (the block's position in its video), or NULL
 *                 meaning block i has index first_block_idx + i.
 *   decisions_out device, n_blocks int32 (1 accept / 0 reject); q_b_out device, n_blocks
 *                 fp32, nullable.
 * Does not synchronise. Returns SDVG_OK or a negative status.
 */
int sdvg_worst_frame_route_batch(const float *frame_scores, int32_t n_blocks, int32_t n_frames,
                                 float tau, const int32_t *block_idx, int32_t first_block_idx,
                                 int32_t *decisions_out, float *q_b_out, void *stream);

/*
 * Average-frame routing, the variant the paper's ablation compares with (Sec. 4.3 "Min-frame
 * vs. average-frame scoring", Table 2): q_b = mean of the block's F per-frame rewards instead
 * of their minimum; everything else (accept iff q_b >= tau, block 0 always rejected, NaN ->
 * reject with q_b = quiet NaN, arguments, return values, synchronisation) as in
 * sdvg_worst_frame_route / _batch. The mean is the fp64 sum of the rewards taken in frame order,
 * divided by F in fp64 and rounded once to fp32, so it is bit-exact against a sequential loop;
 * a mean that comes out NaN (+inf and -inf among the rewards) is reported as the same quiet NaN.
 */
int sdvg_avg_frame_route(const float *frame_scores, int32_t n_frames, float tau, int32_t block_idx,
                         float *q_b_out, void *stream);
int sdvg_avg_frame_route_batch(const float *frame_scores, int32_t n_blocks, int32_t n_frames,
                               float tau, const int32_t *block_idx, int32_t first_block_idx,
                               int32_t *decisions_out, float *q_b_out, void *stream);

/*
 * Measurement aid (no passage of the paper: it exists so that a benchmark can report what the
 * matrix cores of the chip it runs on deliver, next to the attention kernel's rate). Launches
 * 256 workgroups of 4 waves (one wave per SIMD of the chip); every wave issues iters x 16 v_mfma_f32_32x32x16_bf16 from
 * registers and nothing else. Asynchronous on `stream`; the caller times it.
 *   out        device, at least 65536 floats (n_out = its length): checksums, never read back.
 *   cycles     device, one uint64: shader clocks wave 0 took (clock = cycles / measured time).
 *   iters      1 .. 2^24.
 *   flops_out  host, nullable: the FLOPs the launch performs (256 x 4 x iters x 16 x 32768).
 * Returns SDVG_OK or a negative status.
 */
int sdvg_probe_mfma(float *out, int64_t n_out, uint64_t *cycles, int32_t iters, double *flops_out,
                    void *stream);

/*
 * The same measurement with operands that change: the A operand of every MFMA differs from the
 * previous one's and the B operand changes every second MFMA (register sets filled with random
 * signs and mantissas, magnitudes 1/8 .. 4), as the operands of an attention kernel do. The
 * chip holds a lower clock under this load than under sdvg_probe_mfma's, whose two operand
 * registers never change; this is the rate to compare a real kernel with.
 * Arguments, return values and FLOP count as for sdvg_probe_mfma.
 */
int sdvg_probe_mfma_changing(float *out, int64_t n_out, uint64_t *cycles, int32_t iters,
                             double *flops_out, void *stream);

/* Human-readable name of a status code (static storage; never NULL). */
const char *sdvg_status_string(int status);

/* hipError_t of the most recent SDVG_ERR_DEVICE on this thread, as an int (0 if none). */
int sdvg_last_device_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int sdvg_version(void);

/* Releases the small pinned host buffer the router keeps. Safe to call more than once. */
void sdvg_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* SDVG_H */
