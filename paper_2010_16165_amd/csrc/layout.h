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

// One layer of the table, packed into aligned 32-bit words so that the kernel
// reads it with scalar loads only (a byte or unaligned 16-bit field would be
// fetched with a vector load, whose wait would also drain the parameter
// prefetch in flight).
struct ResLayer {             // 48 bytes
  const void* packed;         // conv: blob (bias + weights) in global memory
  uint32_t off0;              // in_org | out_org << 16     LDS offsets, 16-byte units (see below)
  uint32_t off1;              // res_org | w_off << 16      res_org 0xffff = none
  uint32_t sz;                // blob_units | nchunk << 16  blob_units: 16-byte units staged to w_off
  uint32_t ps0;               // ps_in | ps_out << 16       LDS pixel strides, elements
  uint32_t ps1;               // ps_res | cs_out << 16      cs_out: lanes written per output pixel
  uint32_t ch;                // res_cs | Kp << 16          res_cs: lanes held per residual pixel
  uint32_t g0;                // Wh_in | Wh_out << 8 | P << 16 | Q << 24   Wh: pixels per LDS row
  uint32_t g1;                // S | stride << 8 | cpt << 16 | nsteps << 24
  uint32_t g2;                // FT | MT << 8 | NT << 16 | res_Wh << 24    work item: MT x NT tiles
  uint32_t g3;                // res_ss | flags << 8 | out_halo << 16
};
// Tensors in LDS carry a halo of zero pixels.  in_org is the LDS offset of the
// pixel that tap (0, 0) of output pixel (0, 0) reads; out_org and res_org are
// the offsets of interior pixel (0, 0).  For the global-mean layer P x Q is the
// INPUT extent and in_org its interior origin.
static_assert(sizeof(ResLayer) == 48, "ResLayer must stay 48 bytes");
constexpr int kResMean = 1, kResRelu = 2, kResLast = 4;

struct ResParams {
  const void* x;    // N images, NHWC
  void* y;          // N x out_pixels x y_cs
  int in_H, in_W, in_Wh;         // image extent and pixels per LDS row (in_W + 2 * hp)
  int in_cs, in_ps;              // global channel stride, LDS pixel stride (elements)
  int in_org;                    // LDS offset (16-byte units) of the image's interior pixel (0, 0)
  int hp;                        // halo width of every LDS tensor larger than 1 x 1
  int y_cs, out_pixels;
  int n_layers;
  int lds_bytes;
  ResLayer layers[kResMaxLayers];
};
static_assert(sizeof(ResParams) <= 3800, "kernel arguments must stay under 4 KB");

// Each thread carries the next layer's parameters through the current layer
// in kResPrefetch 16-byte registers, so a blob may not exceed this.
constexpr int kResPrefetch = 5;
constexpr size_t kResMaxBlob = (size_t)kResPrefetch * 16 * kResThreads;

fupr_status launch_resident(const ResParams& p, int N, fupr_dtype dt, void* stream);

}  // namespace fupr
