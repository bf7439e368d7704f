// Internal: arguments of the 16-bit implicit-GEMM convolution kernels.
#pragma once
#include <cstdint>

#include "fupr.h"

namespace fupr {

struct Conv16Params {
  const uint16_t* x;
  const uint16_t* w;     // [nchunk_pad][Kp][8]
  const float* bias;     // [Kp]
  const uint16_t* res;
  uint16_t* y;
  int H, W, xcs;
  int P, Q, PQ, M, ycs;
  int S, stride, pad;
  int Kp, FT, cpt, nchunk, nsteps;
  int rH, rW, rcs, rss, roff;
  int relu;
  uint32_t x_bytes, w_bytes;   // extents of x and w, for range-checked buffer loads
  // A block's last convolution after its output filters were pruned (Alg. 1):
  // filter j adds into channel keep[j] of y, which already holds the shortcut,
  // and every other channel of y stays as it is.  keep = nullptr otherwise.
  // keep has keep_n ascending entries in 0 .. yC - 1, in device memory.  Only
  // conv_tiled.hip and conv_patch.hip read these fields.
  const int32_t* keep;
  int keep_n, yC;
  // A second input tensor (fupr_conv_cat_fused, 1 x 1 convolutions only): the
  // 8-channel chunks from `split` on come from x2, read at spatial stride
  // stride2; the chunks before it from x.  x2 = nullptr otherwise.  split is a
  // multiple of 8 (FUPR_CAT_ALIGN channels).  Only conv1x1.hip and conv1x1_pipe.hip read these.
  const uint16_t* x2;
  uint32_t x2_bytes;
  int split, H2, W2, xcs2, stride2;
};

// conv_tiled.hip: LDS-staged filters, register-blocked tiles.  M = N*P*Q.
fupr_status launch_conv16_tiled(const Conv16Params& p, bool bf16, void* stream);
const char* conv16_tiled_name(int FT, int nsteps, int64_t M);

// conv_patch.hip: 3 x 3 convolutions with the workgroup's input patch in LDS.
// Geometry fields of the argument only (H, W, P, Q, PQ, S, stride, pad, cpt,
// nchunk, FT, Kp) and the batch size decide whether it applies and which tile
// it runs.
bool conv_patch_applies(const Conv16Params& geometry, int N);
const char* conv_patch_name(const Conv16Params& geometry, int N);
fupr_status launch_conv_patch(const Conv16Params& p, int N, bool bf16, void* stream);

// conv1x1.hip: 1 x 1 convolutions whose filters fit in LDS, streamed.  Geometry
// fields decide whether it applies.
bool conv1x1_stream_applies(const Conv16Params& geometry);
const char* conv1x1_stream_name(const Conv16Params& geometry);
fupr_status launch_conv1x1_stream(const Conv16Params& p, int N, bool bf16, void* stream);

// conv1x1.hip: a 1 x 1 convolution followed by another 1 x 1 convolution that reads
// all of its output channels, in one launch.
bool conv1x1_fused_pair_applies(const Conv16Params& first, const Conv16Params& second);
fupr_status launch_conv1x1_fused_pair(const Conv16Params& first, const Conv16Params& second, int N,
                                      bool bf16, void* stream);

// conv1x1_pipe.hip: 1 x 1 convolutions with 128 channels or more whose filters do
// not fit in LDS, as a pipelined GEMM.
bool conv1x1_pipe_applies(const Conv16Params& geometry);
const char* conv1x1_pipe_name(const Conv16Params& geometry);
fupr_status launch_conv1x1_pipe(const Conv16Params& p, int N, bool bf16, void* stream);

}  // namespace fupr
