// Two measuring kernels with known work and nothing else, for the roofline
// figures the benchmark reports: the MFMA rate a kernel can reach when it does
// nothing but multiply (in both instruction shapes), and the rate of a plain
// device-to-device copy.  Built into libfupr_measure.so, apart from the product.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "fupr_measure.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Independent accumulators per wave: 16 of 16 x 16 (64 registers), 8 of 32 x 32 (128).
constexpr int kChains16 = 16, kChains32 = 8;

// The instruction stream is written out, so that it is the one measured: chain c
// multiplies operand registers a[c % 4] and b[c / 4 % 4] (a kernel's MFMAs take
// their operands from different registers; a stream that names the same two
// registers in every MFMA was measured at 57 % of this one's rate for 16 x 16 x 32).
template <bool BF, bool WIDE>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float* out) {
  const int lane = threadIdx.x & 63;
  // operands that no compiler can fold: they depend on the lane
  const uint32_t bits = BF ? 0x3f803f80u : 0x3c003c00u;   // two ones
  u32x4 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = u32x4{bits, bits ^ (uint32_t)(lane & 1), bits, bits ^ (uint32_t)(i << 16)};
    b[i] = u32x4{bits, bits, bits ^ (uint32_t)(lane & 2), bits ^ (uint32_t)i};
  }
  float s = 0.f;
  if constexpr (WIDE) {
    f32x16 acc[kChains32];
#pragma unroll
    for (int c = 0; c < kChains32; ++c)
#pragma unroll
      for (int j = 0; j < 16; ++j) acc[c][j] = 0.f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int c = 0; c < kChains32; ++c) {
        if constexpr (BF)
          asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[c]) : "v"(a[c & 3]), "v"(b[(c >> 2) & 3]));
        else
          asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+v"(acc[c]) : "v"(a[c & 3]), "v"(b[(c >> 2) & 3]));
      }
    }
    // the results are read by ordinary instructions: let the last MFMAs finish first
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int c = 0; c < kChains32; ++c)
#pragma unroll
      for (int j = 0; j < 16; ++j) s += acc[c][j];
  } else {
    f32x4 acc[kChains16];
#pragma unroll
    for (int c = 0; c < kChains16; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < iters; ++i) {
#pragma unroll
      for (int c = 0; c < kChains16; ++c) {
        if constexpr (BF)
          asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc[c]) : "v"(a[c & 3]), "v"(b[(c >> 2) & 3]));
        else
          asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc[c]) : "v"(a[c & 3]), "v"(b[(c >> 2) & 3]));
      }
    }
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#pragma unroll
    for (int c = 0; c < kChains16; ++c) s += acc[c][0] + acc[c][1] + acc[c][2] + acc[c][3];
  }
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* src, uint4* dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

int32_t launched() { return hipGetLastError() == hipSuccess ? 0 : -8; }

}  // namespace

extern "C" int32_t fupr_measure_mfma(int32_t dt, int32_t shape, int32_t iters, int32_t workgroups,
                                     void* out, double* flops, void* stream) {
  if (!out || !flops) return -1;
  if (dt != 1 && dt != 2) return -3;
  if ((shape != 16 && shape != 32) || iters <= 0 || workgroups <= 0 || workgroups > (1 << 20)) return -9;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)workgroups), block(256);
  float* o = (float*)out;
  if (dt == 1 && shape == 16) hipLaunchKernelGGL((mfma_rate_kernel<true, false>), grid, block, 0, st, iters, o);
  else if (dt == 1) hipLaunchKernelGGL((mfma_rate_kernel<true, true>), grid, block, 0, st, iters, o);
  else if (shape == 16) hipLaunchKernelGGL((mfma_rate_kernel<false, false>), grid, block, 0, st, iters, o);
  else hipLaunchKernelGGL((mfma_rate_kernel<false, true>), grid, block, 0, st, iters, o);
  // 4 waves per workgroup; per iteration 16 MFMAs of 2 * 16 * 16 * 32 flops or 8 of 2 * 32 * 32 * 16
  *flops = (double)workgroups * 4.0 * iters * (shape == 16 ? kChains16 * 16384.0 : kChains32 * 32768.0);
  return launched();
}

extern "C" int32_t fupr_measure_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return -1;
  if (bytes == 0 || bytes % 16 != 0) return -2;
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return -7;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipLaunchKernelGGL(copy_kernel, dim3(256 * 8), dim3(256), 0, st, (const uint4*)src, (uint4*)dst,
                     bytes / 16);
  return launched();
}
