// Internal: sizes of the packed parameter blob and small helpers shared by the
// host passes, the kernel launchers and the model executor.
#pragma once
#include <cstddef>
#include <cstdint>

#include "fupr.h"

namespace fupr {

inline int round_up(int a, int b) { return (a + b - 1) / b * b; }
inline size_t round_up_sz(size_t a, size_t b) { return (a + b - 1) / b * b; }
inline size_t elem_size(fupr_dtype dt) { return dt == FUPR_F32 ? 4 : 2; }
inline bool dtype_ok(int dt) { return dt == FUPR_F32 || dt == FUPR_BF16 || dt == FUPR_F16; }
inline int c_align(fupr_dtype dt) { return dt == FUPR_F32 ? 4 : 8; }
inline int min_c_stride(int C, fupr_dtype dt) { return round_up(C, c_align(dt)); }
inline int out_extent(int in, int k, int stride, int pad) { return (in + 2 * pad - k) / stride + 1; }

bool shape_ok(const fupr_conv_shape* s);

struct PackedLayout {
  int Kp;          // filters incl. zero padding
  int Cp;          // channels per tap incl. zero padding
  int nchunk;      // 16-bit: R*S*Cp/8 chunks of 8 channels; fp32: R*S*Cp rows
  int nchunk_pad;  // 16-bit: nchunk rounded up to 4; fp32: = nchunk
  size_t weight_offset, total_bytes;
};

inline PackedLayout packed_layout(const fupr_conv_shape& s, fupr_dtype dt) {
  PackedLayout L;
  if (dt == FUPR_F32) {
    L.Kp = round_up(s.K, 4);
    L.Cp = round_up(s.C, 4);
    L.nchunk = L.nchunk_pad = s.R * s.S * L.Cp;
    L.weight_offset = round_up_sz((size_t)L.Kp * 4, 256);
    L.total_bytes = L.weight_offset + (size_t)L.nchunk * L.Kp * 4;
  } else {
    L.Kp = round_up(s.K, 16);
    L.Cp = round_up(s.C, 8);
    L.nchunk = s.R * s.S * (L.Cp / 8);
    L.nchunk_pad = round_up(L.nchunk, 4);
    L.weight_offset = round_up_sz((size_t)L.Kp * 4, 256);
    L.total_bytes = L.weight_offset + (size_t)L.nchunk_pad * L.Kp * 8 * 2;
  }
  L.total_bytes = round_up_sz(L.total_bytes, 256);
  return L;
}

// Launchers (kernels.hip); all arguments already validated.
struct ConvArgs {
  const void* x;
  const void* packed;
  const void* res;
  void* y;
  int N, H, W, C, xcs;   // input
  int P, Q, K, ycs;      // output
  int R, S, stride, pad;
  int rH, rW, rC, rcs, rss, roff;  // residual tensor geometry
  int relu;
  fupr_dtype dt;
};
fupr_status launch_conv(const ConvArgs& a, void* stream);
const char* conv_kernel_name(const fupr_conv_shape& s, fupr_dtype dt, int64_t M);

}  // namespace fupr
