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

// FUPR_OK if the HIP runtime has no pending error, else FUPR_ERR_LAUNCH (the
// runtime's message goes to stderr when the environment has FUPR_DEBUG set).
fupr_status launch_status(const char* what);

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

// ---- whole network in one kernel, activations resident in LDS ----------------
// One workgroup per image walks a table of layers; see resident.hip.

constexpr int kResMaxLayers = 72;
constexpr int kResTableEntries = 256;             // chunks per layer the tap table can hold
constexpr int kResThreads = 1024;
constexpr size_t kResLdsLimit = 160 * 1024;

struct ResLayer {             // 48 bytes
  const void* packed;         // conv: blob (bias + weights)
  uint16_t in_off, out_off, res_off;  // LDS offsets in 16-byte units; res_off 0xffff = none
  uint16_t nchunk;
  uint16_t cs_in, cs_out, res_cs;     // elements per pixel
  uint16_t Kp;
  uint8_t kind;               // 0 conv, 1 global mean
  uint8_t H, W, P, Q;
  uint8_t S, stride, pad;
  uint8_t cpt, nsteps, FT, NT;
  uint8_t res_W, res_ss;
  uint8_t relu, last;
  uint8_t reserved[4];
};
static_assert(sizeof(ResLayer) == 48, "ResLayer must stay 48 bytes");

struct ResParams {
  const void* x;    // N images, NHWC, in_elems elements each
  void* y;          // N x out_pixels x y_cs
  int in_elems;     // per image
  int in_off;       // LDS offset (16-byte units) the image is staged to
  int y_cs, out_pixels;
  int n_layers;
  int lds_bytes;
  ResLayer layers[kResMaxLayers];
};
static_assert(sizeof(ResParams) <= 3800, "kernel arguments must stay under 4 KB");

fupr_status launch_resident(const ResParams& p, int N, fupr_dtype dt, void* stream);

}  // namespace fupr
