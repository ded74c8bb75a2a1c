// Launch parameters shared by the attention kernels (internal to libsdvg).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sdvg {

constexpr int kMaxAttnItems = 8;  // (q, cache, block, out) sets one launch can take

struct AttnItem {
  const void *q, *k_cache, *v_cache, *k_blk, *v_blk;
  void *out;
};

struct AttnParams {
  AttnItem items[kMaxAttnItems];
  int64_t q_ts, q_hs, o_ts, o_hs, kv_ts, kv_hs, blk_ts, blk_hs;  // strides in elements
  int64_t cache_len;
  float *partials;    // partial results of query tiles whose keys are split over workgroups (or null)
  // fused commit: workgroups past the attention work copy item 0's block into these rows (or null)
  void *k_commit_dst, *v_commit_dst;
  int32_t n_blk, copy_first_block, n_copy_blocks;
  int32_t n_items, n_q, n_k, n_heads, n_qtiles;
  int32_t n_hq;       // query tiles of the launch: n_items * n_heads * n_qtiles
  int32_t n_tiles;    // key tiles: ceil(n_k / 64)
  int32_t units;      // (query tile, key tile) pairs per workgroup; == n_tiles when nothing is split
  int32_t total_work; // workgroups with work
  int32_t work_per_xcd;
  int32_t wt_base, wt_rem;  // 32-row wave tiles per workgroup: wt_base, plus one for the first wt_rem
  float scale_log2e;  // scale * log2(e)
};

// Floats one workgroup writes per partial result: 8 waves x (64 accumulators + row sum + shift) x 64 lanes.
constexpr int64_t kPartialFloats = 8 * 66 * 64;

// fp32 check path (block_attn_f32.hip): same mathematics, fp32 inputs / P / output; item 0 only.
int launch_block_attn_f32(const AttnParams &p, hipStream_t stream);

}  // namespace sdvg
