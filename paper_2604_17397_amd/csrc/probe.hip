// Measurement aid, not a step of the paper's method: a kernel that does nothing but bf16 MFMAs
// from registers, so that a benchmark can put the attention kernel's rate next to what the
// matrix pipes of THIS chip deliver at the clock it settles at under such a load (the 2.5
// PFLOP/s datasheet peak assumes 2.4 GHz, which an MI355X does not hold under matrix load).
#include <stdint.h>

#include "sdvg.h"
#include "sdvg_common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kProbeGroups = 256;  // one workgroup per CU, one wave per SIMD
constexpr int kProbeMfmaPerIter = 16;

// Every wave issues iters x 16 v_mfma_f32_32x32x16_bf16 on four independent accumulators.
// out[2 * wave_global] = accumulator checksum, so that nothing is optimised away; lane 0 of
// wave 0 of workgroup 0 also stores its elapsed shader clocks in cycles[0].
// kChanging = false: every MFMA reads the same two operand registers (few mantissa bits set):
// the matrix pipes at their lowest switching energy. kChanging = true: the A operand differs
// from one MFMA to the next (eight register sets in turn) and the B operand every second one
// (four sets), all with random signs and mantissas and magnitudes 1/8 .. 4, which is how the
// operands of an attention kernel arrive; the chip's clock under that load is the one a real
// kernel can hope for.
template <bool kChanging>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *out, unsigned long long *cycles, int iters) {
  const int lane = threadIdx.x & 63;
  constexpr int kNa = kChanging ? 8 : 1, kNb = kChanging ? 4 : 1;
  bf16x8 a[kNa], b[kNb];
  if constexpr (kChanging) {
    uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
    auto draw = [&]() {
      h ^= h << 13;
      h ^= h >> 17;
      h ^= h << 5;
      const uint16_t bits =
          static_cast<uint16_t>(((h >> 3) & 0x8000u) | ((124u + ((h >> 8) % 6u)) << 7) | (h & 0x7fu));
      __bf16 r;
      __builtin_memcpy(&r, &bits, 2);
      return r;
    };
#pragma unroll
    for (int n = 0; n < kNa; ++n)
#pragma unroll
      for (int i = 0; i < 8; ++i) a[n][i] = draw();
#pragma unroll
    for (int n = 0; n < kNb; ++n)
#pragma unroll
      for (int i = 0; i < 8; ++i) b[n][i] = draw();
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[0][i] = static_cast<__bf16>(0.03125f * static_cast<float>((lane * 7 + i * 3) % 17 - 8));
      b[0][i] = static_cast<__bf16>(0.015625f * static_cast<float>((lane * 5 + i) % 13 - 6));
    }
  }
  f32x16 c[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[n][i] = 0.f;
  const unsigned long long t0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < kProbeMfmaPerIter; ++m)
      c[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m % kNa], b[(m / 2) % kNb], c[m & 3], 0, 0, 0);
  }
  float r = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += c[n][i];
  const unsigned long long t1 = __builtin_readcyclecounter();
  out[blockIdx.x * 256 + threadIdx.x] = r;
  if (blockIdx.x == 0 && threadIdx.x == 0) cycles[0] = t1 - t0;
}

int launch_probe(bool changing, float *out, int64_t n_out, uint64_t *cycles, int32_t iters, double *flops_out,
                 void *stream) {
  if (!out || !cycles) return SDVG_ERR_NULL;
  if (n_out < int64_t{kProbeGroups} * 256) return SDVG_ERR_SHAPE;
  if (iters < 1 || iters > (1 << 24)) return SDVG_ERR_RANGE;
  auto *cyc = reinterpret_cast<unsigned long long *>(cycles);
  if (changing)
    hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(kProbeGroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       out, cyc, iters);
  else
    hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(kProbeGroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       out, cyc, iters);
  SDVG_HIP_CHECK(hipGetLastError());
  if (flops_out)
    *flops_out = static_cast<double>(kProbeGroups) * 4.0 * iters * kProbeMfmaPerIter * (2.0 * 32 * 32 * 16);
  return SDVG_OK;
}

}  // namespace

extern "C" int sdvg_probe_mfma(float *out, int64_t n_out, uint64_t *cycles, int32_t iters,
                               double *flops_out, void *stream) {
  return launch_probe(false, out, n_out, cycles, iters, flops_out, stream);
}

extern "C" int sdvg_probe_mfma_changing(float *out, int64_t n_out, uint64_t *cycles, int32_t iters,
                                        double *flops_out, void *stream) {
  return launch_probe(true, out, n_out, cycles, iters, flops_out, stream);
}
