// Internal: 16-bit element conversion and MFMA wrappers shared by the kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace fupr {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <bool BF>
__device__ __forceinline__ float to_float(uint16_t h) {
  if constexpr (BF) {
    return __uint_as_float((uint32_t)h << 16);
  } else {
    return (float)__builtin_bit_cast(_Float16, h);
  }
}

// Round to nearest even.
template <bool BF>
__device__ __forceinline__ uint16_t from_float(float f) {
  if constexpr (BF) {
    return __builtin_bit_cast(uint16_t, (__bf16)f);   // v_cvt_pk_bf16_f32 on gfx950
  } else {
    return __builtin_bit_cast(uint16_t, (_Float16)f);
  }
}

// Two floats rounded to nearest even and packed, a in the low half.
template <bool BF>
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {a, b};
  if constexpr (BF) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  } else {
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
  }
}

template <bool BF>
__device__ __forceinline__ f32x4 mfma_16x16x32(const uint4& a, const uint4& b, f32x4 c) {
  if constexpr (BF) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
}

// D (32 x 32) += A (32 x 16) * B (16 x 32).  Lane l holds row l % 32 of A and column
// l % 32 of B, reduction indices 8 * (l / 32) .. + 7 of each; of D it holds column
// l % 32, rows 8 * (v / 4) + 4 * (l / 32) + v % 4 in element v.  Both shapes sustain
// the full MFMA rate on gfx950 (measured: 2.47 PFLOP/s); this one moves half as many
// operand bytes per flop at the same tile size per instruction.
template <bool BF>
__device__ __forceinline__ f32x16 mfma_32x32x16(const uint4& a, const uint4& b, f32x16 c) {
  if constexpr (BF) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
}

// floor(v / d) for 0 <= v < 2^31 as mulhi(v, mul) >> shift with shift =
// ceil(log2 d) - 1, mul = ceil(2^(32 + shift) / d) < 2^32 (the error mul * d -
// 2^(32 + shift) is below d <= 2^(shift + 1), hence exact while v < 2^31);
// mul = 0 stands for d = 1.
struct FastDiv {
  uint32_t mul, shift;
};

__device__ __forceinline__ int div_by(int v, const FastDiv& d) {
  const uint32_t q = __umulhi((uint32_t)v, d.mul) >> d.shift;
  return d.mul ? (int)q : v;
}

inline FastDiv fast_div(int d) {
  if (d <= 1) return FastDiv{0u, 0u};
  uint32_t shift = 0;
  while ((1u << (shift + 1)) < (uint32_t)d) ++shift;   // ceil(log2 d) - 1
  const uint64_t two = uint64_t(1) << (32 + shift);
  return FastDiv{(uint32_t)((two + (uint64_t)d - 1) / (uint64_t)d), shift};
}

}  // namespace fupr
