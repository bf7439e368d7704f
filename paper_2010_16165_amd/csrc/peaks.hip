// Two measuring kernels with known work and nothing else, for the roofline
// figures the benchmark reports: the MFMA rate a kernel can reach when it does
// nothing but multiply, and the rate of a plain device-to-device copy.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "device_utils.h"
#include "fupr.h"
#include "layout.h"

namespace fupr {
namespace {

constexpr int kChains = 8;   // independent accumulators per wave

template <bool BF>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float* out) {
  const int lane = threadIdx.x & 63;
  // operands that no compiler can fold: they depend on the lane
  const uint32_t bits = BF ? 0x3f803f80u : 0x3c003c00u;   // two ones
  const uint4 a = {bits, bits ^ (uint32_t)(lane & 1), bits, bits};
  const uint4 b = {bits, bits, bits ^ (uint32_t)(lane & 2), bits};
  f32x4 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int c = 0; c < kChains; ++c) acc[c] = mfma_16x16x32<BF>(a, b, acc[c]);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* src, uint4* dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace
}  // namespace fupr

using namespace fupr;

extern "C" fupr_status fupr_measure_mfma(int32_t dt, int32_t iters, int32_t workgroups, void* out,
                                         double* flops, void* stream) {
  if (!out || !flops) return FUPR_ERR_NULL;
  if (dt != FUPR_BF16 && dt != FUPR_F16) return FUPR_ERR_DTYPE;
  if (iters <= 0 || workgroups <= 0 || workgroups > (1 << 20)) return FUPR_ERR_ARG;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (dt == FUPR_BF16)
    hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3((unsigned)workgroups), dim3(256), 0, st, iters,
                       (float*)out);
  else
    hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3((unsigned)workgroups), dim3(256), 0, st, iters,
                       (float*)out);
  // 4 waves per workgroup, kChains MFMAs of 16 x 16 x 32 (2 * 16 * 16 * 32 flops) per iteration
  *flops = (double)workgroups * 4.0 * iters * kChains * 2.0 * 16 * 16 * 32;
  return launch_status("mfma_rate_kernel");
}

extern "C" fupr_status fupr_measure_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return FUPR_ERR_NULL;
  if (bytes == 0 || bytes % 16 != 0) return FUPR_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return FUPR_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(copy_kernel, dim3(256 * 8), dim3(256), 0, st, (const uint4*)src, (uint4*)dst,
                     bytes / 16);
  return launch_status("copy_kernel");
}
