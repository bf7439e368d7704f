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
  const int32_t* keep;   // device, K entries: filter j adds into channel keep[j] of y; else nullptr
  int yC;                // with keep: channels of y
  // second input of a convolution over two concatenated tensors; x2 = nullptr otherwise
  const void* x2;
  int H2, W2, xcs2, stride2;
  int split_c;           // input channels taken from x (a multiple of 32); the others come from x2
};
fupr_status launch_conv(const ConvArgs& a, void* stream);
// indexed: the convolution adds into listed channels of a wider tensor (ConvArgs::keep)
const char* conv_kernel_name(const fupr_conv_shape& s, fupr_dtype dt, int N, int H, int W,
                             bool indexed = false, bool two_inputs = false);
// fupr_conv_cat_fused followed by a 1 x 1 convolution of its output, in one launch
// (what fupr_conv_conv1x1_fused is to fupr_conv_fused); for the model executor.
fupr_status conv_cat_conv1x1_fused(const fupr_conv_shape* shape1, const fupr_tensor* x1,
                                   const fupr_tensor* x2, int32_t x2_stride, const void* packed1,
                                   uint32_t flags1, const fupr_tensor* y,
                                   const fupr_conv_shape* shape2, const void* packed2,
                                   uint32_t flags2, const fupr_tensor* h, void* stream);
// Shapes only: can convolution s1 on an N x H x W input and convolution s2 on its
// output run as one launch (fupr_conv_conv1x1_fused)?
bool conv_pair_fusable(const fupr_conv_shape& s1, const fupr_conv_shape& s2, fupr_dtype dt, int N,
                       int H, int W);

// ---- whole network in one kernel, activations resident in LDS ----------------
// One workgroup per image walks a table of layers; see resident.hip.

constexpr int kResMaxLayers = 256;
constexpr int kResThreads = 1024;
constexpr size_t kResLdsLimit = 160 * 1024;
constexpr int kResScratchBytes = 2048;            // start of LDS: partial sums of the mean layer

// One layer of the table the kernel walks (device memory, read with scalar
// loads).  Everything the kernel would otherwise derive per layer is worked out
// once on the host: LDS byte offsets, byte strides per output row / column,
// reciprocal multipliers for the two divisions, the work-item count.
//
// Tensors in LDS carry a halo of zero pixels.  in_org is the LDS byte offset of
// the pixel that tap (0, 0) of output pixel (0, 0) reads (the tap table's entries
// include it); out_org and res_org
// are the offsets of interior pixel (0, 0).  For the global-mean layer M is the
// INPUT pixel count, Q its width, in_org its interior origin, in_row / in_col
// its byte strides.
struct ResLayer {
  const void* packed;        // conv: blob (bias + weights) in global memory
  const void* table;         // conv: tap table in global memory, (nsteps + kResTablePad) * 4 LDS byte offsets
  int32_t blob_units;        // 16-byte units staged to w_off
  int32_t tab_units;         // 16-byte units staged to tab_off
  int32_t w_off, tab_off;    // LDS byte offsets of the blob and of the table
  int32_t wts_off, wstep;    // LDS byte offset of the weights; bytes per MFMA step (4 chunks)
  int32_t in_org, out_org, res_org;   // res_org < 0: no shortcut
  int32_t in_row, in_col;    // bytes from an output pixel's window to the next row's / column's
  int32_t out_row, out_col, res_row, res_col;
  int32_t M, Q;              // output pixels, output width
  uint32_t magicQ;           // floor(m / Q) = mulhi(m, magicQ) for m < 2^16; 0 when Q = 1
  uint32_t magicF;           // floor(item / n_fgroups), likewise
  int32_t nsteps, FT;        // MFMA steps along (r, s, c); filter tiles of 16
  int32_t MT, NT;            // work item: MT pixel tiles x NT filter tiles
  int32_t n_fgroups, n_items;
  int32_t cs_out, res_cs;    // lanes written per output pixel, lanes held per shortcut pixel
  int32_t flags;
  // halo of the output tensor, zeroed by this layer when kResZeroHalo is set
  int32_t hz_org, hz_P, hz_Q, hz_Wh, hz_ps2, hz_chunks, hz_hp;
  int32_t pad_[1];
  // what staging the NEXT layer's parameters needs (a copy of that layer's first
  // eight dwords), so that no load stands between a layer's start and the staging
  const void* next_packed;
  const void* next_table;
  int32_t next_blob_units, next_tab_units, next_w_off, next_tab_off;
};
static_assert(sizeof(ResLayer) == 192, "ResLayer is read as 48 dwords");
constexpr int kResMean = 1, kResRelu = 2, kResLast = 4, kResZeroHalo = 8;
// kResFullPixels: the pixel count is a multiple of a work item's pixels (no
// clamped pixel).  kResFullFilters: no work item has a missing filter tile and
// all 16 lanes of every filter tile are stored.  kResReuse: a wave's first work
// item covers the same pixels at the same strides as in the previous conv
// layer, no pixel tile is ragged, and the output's strides are the input's.
// kResLikeOut: the shortcut tensor has the output's strides.
constexpr int kResFullPixels = 16, kResReuse = 32, kResLikeOut = 64, kResFullFilters = 128;
// An entry with n_items = 0 and no flag is not a layer of the network: it only
// stages the parameters of the entry after it (no wave has a work item, so all
// stage).  The planner puts one in front of a layer whose parameters find no
// room in LDS during the layer before it.
constexpr int kResTablePad = 8;   // steps of padding after a tap table (2 * deepest prefetch)

struct ResParams {
  const void* x;             // N images, NHWC
  void* y;                   // N x out_pixels x y_cs
  const ResLayer* layers;    // device memory
  int in_H, in_W, in_Wh;     // image extent and pixels per LDS row (in_W + 2 * hp)
  int in_cs, in_ps2;         // global channel stride (elements), LDS pixel stride (bytes)
  int in_org;                // LDS byte offset of the image's interior pixel (0, 0)
  int hp;                    // halo width of every LDS tensor larger than 1 x 1
  int y_cs, out_pixels;
  int n_layers;
  int lds_bytes;
};

fupr_status launch_resident(const ResParams& p, int N, fupr_dtype dt, void* stream);

}  // namespace fupr
