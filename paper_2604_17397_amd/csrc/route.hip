// Worst-frame routing: q_b = min over a block's per-frame rewards (paper Sec. 3 Eq. (1)),
// accept iff q_b >= tau ("Inference flow"), block 0 always rejected ("Force-reject the first
// block"). One wavefront per video block; the single-block call writes its result into pinned
// host memory and waits for the stream, because the caller branches on the decision.
#include <mutex>

#include "sdvg_common.h"

namespace {

constexpr int kWave = 64;
constexpr uint32_t kQuietNaN = 0x7FC00000u;

// Order-preserving map float bits -> unsigned key: more negative floats get smaller keys and
// -0.0 sorts just below +0.0, so the minimum key is unique whatever the reduction order.
__device__ __forceinline__ uint32_t order_key(uint32_t bits) {
  return (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
}
__device__ __forceinline__ uint32_t key_to_bits(uint32_t key) {
  return (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;
}

__global__ __launch_bounds__(kWave) void worst_frame_route_kernel(
    const float *__restrict__ scores, int n_frames, float tau, const int32_t *__restrict__ block_idx,
    int first_block_idx, int32_t *__restrict__ decisions, float *__restrict__ q_b) {
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  const float *s = scores + static_cast<int64_t>(b) * n_frames;
  uint32_t key = 0xFFFFFFFFu;  // above every real key (that pattern maps back to a NaN)
  int has_nan = 0;
  for (int i = lane; i < n_frames; i += kWave) {
    const uint32_t bits = __float_as_uint(s[i]);
    has_nan |= ((bits & 0x7FFFFFFFu) > 0x7F800000u);
    const uint32_t k = order_key(bits);
    key = k < key ? k : key;
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {
    const uint32_t other = __shfl_xor(key, off, kWave);
    key = other < key ? other : key;
    has_nan |= __shfl_xor(has_nan, off, kWave);
  }
  if (lane == 0) {
    const int idx = block_idx ? block_idx[b] : first_block_idx + b;
    const uint32_t bits = has_nan ? kQuietNaN : key_to_bits(key);
    const float qb = __uint_as_float(bits);
    decisions[b] = (!has_nan && idx != 0 && qb >= tau) ? 1 : 0;
    if (q_b) q_b[b] = qb;
  }
}

// Average-frame variant (the paper's ablation "Min-frame vs. average-frame scoring", Table 2):
// q_b = mean of the block's per-frame rewards. One THREAD per video block adds the rewards in
// frame order in fp64 and divides in fp64, so the result does not depend on any reduction order
// and matches a sequential host loop bit for bit.
__global__ __launch_bounds__(kWave) void avg_frame_route_kernel(
    const float *__restrict__ scores, int n_blocks, int n_frames, float tau,
    const int32_t *__restrict__ block_idx, int first_block_idx, int32_t *__restrict__ decisions,
    float *__restrict__ q_b) {
  const int b = blockIdx.x * kWave + threadIdx.x;
  if (b >= n_blocks) return;
  const float *s = scores + static_cast<int64_t>(b) * n_frames;
  double acc = 0.0;
  int has_nan = 0;
  for (int i = 0; i < n_frames; ++i) {
    const float v = s[i];
    has_nan |= ((__float_as_uint(v) & 0x7FFFFFFFu) > 0x7F800000u);
    acc += static_cast<double>(v);
  }
  const int idx = block_idx ? block_idx[b] : first_block_idx + b;
  float qb = static_cast<float>(acc / static_cast<double>(n_frames));
  if (has_nan || qb != qb) qb = __uint_as_float(kQuietNaN);  // (+inf and -inf among the scores sum to NaN)
  decisions[b] = (idx != 0 && qb >= tau) ? 1 : 0;
  if (q_b) q_b[b] = qb;
}

struct RouteResult {
  int32_t decision;
  float q_b;
};
std::mutex g_route_mutex;
RouteResult *g_route_result = nullptr;  // pinned host memory, device-visible

int launch(const float *scores, int n_blocks, int n_frames, float tau, const int32_t *block_idx,
           int first_block_idx, int32_t *decisions, float *q_b, hipStream_t s, bool mean = false) {
  if (mean)
    hipLaunchKernelGGL(avg_frame_route_kernel, dim3((n_blocks + kWave - 1) / kWave), dim3(kWave), 0, s, scores,
                       n_blocks, n_frames, tau, block_idx, first_block_idx, decisions, q_b);
  else
    hipLaunchKernelGGL(worst_frame_route_kernel, dim3(n_blocks), dim3(kWave), 0, s, scores, n_frames,
                       tau, block_idx, first_block_idx, decisions, q_b);
  SDVG_HIP_CHECK(hipGetLastError());
  return SDVG_OK;
}

}  // namespace

namespace {
int route_single(const float *frame_scores, int32_t n_frames, float tau, int32_t block_idx, float *q_b_out,
                 void *stream, bool mean) {
  if (!frame_scores) return SDVG_ERR_NULL;
  if (n_frames < 1) return SDVG_ERR_SHAPE;
  if (tau != tau || block_idx < 0) return SDVG_ERR_RANGE;
  if (reinterpret_cast<uintptr_t>(frame_scores) & 3u) return SDVG_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  std::lock_guard<std::mutex> lock(g_route_mutex);
  if (!g_route_result) {
    void *p = nullptr;
    SDVG_HIP_CHECK(hipHostMalloc(&p, sizeof(RouteResult), hipHostMallocDefault));
    g_route_result = static_cast<RouteResult *>(p);
  }
  g_route_result->decision = -1;
  int st = launch(frame_scores, 1, n_frames, tau, nullptr, block_idx, &g_route_result->decision,
                  &g_route_result->q_b, s, mean);
  if (st != SDVG_OK) return st;
  SDVG_HIP_CHECK(hipStreamSynchronize(s));
  if (q_b_out) *q_b_out = g_route_result->q_b;
  return g_route_result->decision;
}

int route_batch(const float *frame_scores, int32_t n_blocks, int32_t n_frames, float tau,
                const int32_t *block_idx, int32_t first_block_idx, int32_t *decisions_out, float *q_b_out,
                void *stream, bool mean) {
  if (!frame_scores || !decisions_out) return SDVG_ERR_NULL;
  if (n_frames < 1 || n_blocks < 1) return SDVG_ERR_SHAPE;
  if (tau != tau || (!block_idx && first_block_idx < 0)) return SDVG_ERR_RANGE;
  if (reinterpret_cast<uintptr_t>(frame_scores) & 3u) return SDVG_ERR_ALIGN;
  return launch(frame_scores, n_blocks, n_frames, tau, block_idx, first_block_idx, decisions_out,
                q_b_out, static_cast<hipStream_t>(stream), mean);
}
}  // namespace

extern "C" int sdvg_worst_frame_route(const float *frame_scores, int32_t n_frames, float tau,
                                      int32_t block_idx, float *q_b_out, void *stream) {
  return route_single(frame_scores, n_frames, tau, block_idx, q_b_out, stream, false);
}

extern "C" int sdvg_worst_frame_route_batch(const float *frame_scores, int32_t n_blocks,
                                            int32_t n_frames, float tau, const int32_t *block_idx,
                                            int32_t first_block_idx, int32_t *decisions_out,
                                            float *q_b_out, void *stream) {
  return route_batch(frame_scores, n_blocks, n_frames, tau, block_idx, first_block_idx, decisions_out,
                     q_b_out, stream, false);
}

extern "C" int sdvg_avg_frame_route(const float *frame_scores, int32_t n_frames, float tau,
                                    int32_t block_idx, float *q_b_out, void *stream) {
  return route_single(frame_scores, n_frames, tau, block_idx, q_b_out, stream, true);
}

extern "C" int sdvg_avg_frame_route_batch(const float *frame_scores, int32_t n_blocks, int32_t n_frames,
                                          float tau, const int32_t *block_idx, int32_t first_block_idx,
                                          int32_t *decisions_out, float *q_b_out, void *stream) {
  return route_batch(frame_scores, n_blocks, n_frames, tau, block_idx, first_block_idx, decisions_out,
                     q_b_out, stream, true);
}

extern "C" void sdvg_shutdown(void) {
  std::lock_guard<std::mutex> lock(g_route_mutex);
  if (g_route_result) {
    (void)hipHostFree(g_route_result);
    g_route_result = nullptr;
  }
}
