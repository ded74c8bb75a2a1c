// Internal helpers shared by the translation units of libsdvg (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sdvg.h"

namespace sdvg {

// hipError_t of the last failed runtime call on this thread (sdvg_last_device_error()).
extern thread_local int g_last_device_error;

inline int device_error(hipError_t e) {
  g_last_device_error = static_cast<int>(e);
  return SDVG_ERR_DEVICE;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// kv_cache.hip: host-side checks shared by every commit entry point.
int check_commit_args(const sdvg_kv_cache *cache, const void *k_blk, const void *v_blk, int32_t slot);

}  // namespace sdvg

#define SDVG_HIP_CHECK(expr)                                   \
  do {                                                         \
    hipError_t sdvg_e_ = (expr);                               \
    if (sdvg_e_ != hipSuccess) return sdvg::device_error(sdvg_e_); \
  } while (0)
