// Launch parameters shared by the attention kernels (internal to libsdvg).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sdvg {

struct AttnParams {
  const void *q, *k_cache, *v_cache, *k_blk, *v_blk;
  void *out;
  int64_t q_ts, q_hs, o_ts, o_hs, kv_ts, kv_hs, blk_ts, blk_hs;  // strides in elements
  int64_t cache_len;
  int32_t n_q, n_k, n_heads, n_qtiles, total_work, work_per_xcd;
  int32_t wt_base, wt_rem;  // 32-row wave tiles per workgroup: wt_base, plus one for the first wt_rem
  float scale_log2e;  // scale * log2(e)
};

// fp32 check path (block_attn_f32.hip): same mathematics, fp32 inputs / P / output.
int launch_block_attn_f32(const AttnParams &p, hipStream_t stream);

}  // namespace sdvg
