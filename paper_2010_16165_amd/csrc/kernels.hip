// Device kernels for gfx950 and the C-ABI calls that launch them:
// the convolution operator with fused epilogue (Sec. III; Sec. IV-B-1 of the
// paper), max-pool and global mean (the "Others" of Table II).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "fupr.h"
#include "layout.h"
#include "tuning.h"
#include "stem_pool.h"
#include "device_utils.h"
#include "conv16.h"

namespace fupr {
namespace {

// ---- fp32 direct convolution ------------------------------------------------
// One thread: one output pixel x 4 consecutive filters, plain FMA.

struct Conv32Params {
  const float* x;
  const float* w;   // [R*S*Cp][Kp]
  const float* bias;
  const float* res;
  float* y;
  int H, W, xcs, Cp;
  int P, Q, PQ, M, ycs;
  int R, S, stride, pad;
  int Kp, KQ;
  int rH, rW, rcs, rss, roff;
  int relu;
};

__global__ __launch_bounds__(256) void conv32_kernel(const Conv32Params p) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int kq = (int)(idx % p.KQ);
  const int64_t m64 = idx / p.KQ;
  if (m64 >= p.M) return;
  const int m = (int)m64;
  const int k0 = kq * 4;
  const int n = m / p.PQ, rem = m - n * p.PQ;
  const int pp = rem / p.Q, qq = rem - pp * p.Q;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int r = 0; r < p.R; ++r) {
    const int ih = pp * p.stride + r - p.pad;
    if (ih < 0 || ih >= p.H) continue;
    for (int s = 0; s < p.S; ++s) {
      const int iw = qq * p.stride + s - p.pad;
      if (iw < 0 || iw >= p.W) continue;
      const float* xp = p.x + (((int64_t)n * p.H + ih) * p.W + iw) * p.xcs;
      const float* wp = p.w + (size_t)(r * p.S + s) * p.Cp * p.Kp + k0;
      for (int c = 0; c < p.Cp; c += 4) {
        const float4 xv = *reinterpret_cast<const float4*>(xp + c);
        const float xs[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float4 wv = *reinterpret_cast<const float4*>(wp + (size_t)(c + i) * p.Kp);
          acc[0] = fmaf(xs[i], wv.x, acc[0]);
          acc[1] = fmaf(xs[i], wv.y, acc[1]);
          acc[2] = fmaf(xs[i], wv.z, acc[2]);
          acc[3] = fmaf(xs[i], wv.w, acc[3]);
        }
      }
    }
  }
  if (k0 >= p.ycs) return;
  const float4 b4 = *reinterpret_cast<const float4*>(p.bias + k0);
  float v[4] = {acc[0] + b4.x, acc[1] + b4.y, acc[2] + b4.z, acc[3] + b4.w};
  if (p.res) {
    const int kk = k0 - p.roff;
    if (kk >= 0 && kk < p.rcs) {
      const float4 rv = *reinterpret_cast<const float4*>(
          p.res + (((int64_t)n * p.rH + pp * p.rss) * p.rW + qq * p.rss) * p.rcs + kk);
      v[0] += rv.x;
      v[1] += rv.y;
      v[2] += rv.z;
      v[3] += rv.w;
    }
  }
  if (p.relu) {
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
  }
  *reinterpret_cast<float4*>(p.y + (int64_t)m * p.ycs + k0) = float4{v[0], v[1], v[2], v[3]};
}

// ---- pools -------------------------------------------------------------------

struct PoolParams {
  const void* x;
  void* y;
  int H, W, cs, P, Q, ycs, k, stride, pad;
  int chunks;      // channel chunks per pixel that are processed (of the OUTPUT stride)
  int64_t total;   // threads
};

// DT: 0 fp32 (chunk = 4 channels), 1 bf16, 2 fp16 (chunk = 8 channels).
template <int DT>
__global__ __launch_bounds__(256) void maxpool_kernel(const PoolParams p) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= p.total) return;
  const int ch = (int)(idx % p.chunks);
  int64_t pix = idx / p.chunks;
  const int q = (int)(pix % p.Q);
  pix /= p.Q;
  const int pp = (int)(pix % p.P);
  const int n = (int)(pix / p.P);
  constexpr int V = DT == 0 ? 4 : 8;
  float m[V];
#pragma unroll
  for (int i = 0; i < V; ++i) m[i] = -INFINITY;
  for (int r = 0; r < p.k; ++r) {
    const int ih = pp * p.stride + r - p.pad;
    if (ih < 0 || ih >= p.H) continue;
    for (int s = 0; s < p.k; ++s) {
      const int iw = q * p.stride + s - p.pad;
      if (iw < 0 || iw >= p.W) continue;
      const int64_t off = (((int64_t)n * p.H + ih) * p.W + iw) * p.cs + ch * V;
      if constexpr (DT == 0) {
        const float4 v = *reinterpret_cast<const float4*>((const float*)p.x + off);
        m[0] = fmaxf(m[0], v.x);
        m[1] = fmaxf(m[1], v.y);
        m[2] = fmaxf(m[2], v.z);
        m[3] = fmaxf(m[3], v.w);
      } else {
        const uint4 v = *reinterpret_cast<const uint4*>((const uint16_t*)p.x + off);
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          m[2 * i] = fmaxf(m[2 * i], to_float<DT == 1>((uint16_t)(u[i] & 0xffffu)));
          m[2 * i + 1] = fmaxf(m[2 * i + 1], to_float<DT == 1>((uint16_t)(u[i] >> 16)));
        }
      }
    }
  }
  const int64_t yoff = (((int64_t)n * p.P + pp) * p.Q + q) * p.ycs + ch * V;
  if constexpr (DT == 0) {
    *reinterpret_cast<float4*>((float*)p.y + yoff) = float4{m[0], m[1], m[2], m[3]};
  } else {
    uint4 o;
    uint32_t u[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      u[i] = (uint32_t)from_float<DT == 1>(m[2 * i]) |
             ((uint32_t)from_float<DT == 1>(m[2 * i + 1]) << 16);
    o.x = u[0];
    o.y = u[1];
    o.z = u[2];
    o.w = u[3];
    *reinterpret_cast<uint4*>((uint16_t*)p.y + yoff) = o;
  }
}

// Global mean.  A workgroup is 32 (image, channel chunk) pairs x 8 parts: part k
// sums pixels k, k + 8, ... in fp32, the 8 partial sums are then added in order.
constexpr int kPoolParts = 8;
template <int DT>
__global__ __launch_bounds__(256) void avgpool_kernel(const PoolParams p) {
  constexpr int V = DT == 0 ? 4 : 8;
  __shared__ float partial[kPoolParts][32][V];
  const int slot = threadIdx.x & 31, part = threadIdx.x >> 5;
  const int64_t idx = (int64_t)blockIdx.x * 32 + slot;
  const bool live = idx < p.total;
  const int ch = live ? (int)(idx % p.chunks) : 0;
  const int n = live ? (int)(idx / p.chunks) : 0;
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.f;
  const int hw = p.H * p.W;
  for (int i = part; live && i < hw; i += kPoolParts) {
    const int64_t off = ((int64_t)n * hw + i) * p.cs + ch * V;
    if constexpr (DT == 0) {
      const float4 v = *reinterpret_cast<const float4*>((const float*)p.x + off);
      acc[0] += v.x;
      acc[1] += v.y;
      acc[2] += v.z;
      acc[3] += v.w;
    } else {
      const uint4 v = *reinterpret_cast<const uint4*>((const uint16_t*)p.x + off);
      const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc[2 * j] += to_float<DT == 1>((uint16_t)(u[j] & 0xffffu));
        acc[2 * j + 1] += to_float<DT == 1>((uint16_t)(u[j] >> 16));
      }
    }
  }
#pragma unroll
  for (int i = 0; i < V; ++i) partial[part][slot][i] = acc[i];
  __syncthreads();
  if (part != 0 || !live) return;
#pragma unroll
  for (int i = 0; i < V; ++i) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < kPoolParts; ++k) s += partial[k][slot][i];
    acc[i] = s;
  }
  const float inv = (float)hw;
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = acc[i] / inv;
  const int64_t yoff = (int64_t)n * p.ycs + ch * V;
  if constexpr (DT == 0) {
    *reinterpret_cast<float4*>((float*)p.y + yoff) = float4{acc[0], acc[1], acc[2], acc[3]};
  } else {
    uint4 o;
    uint32_t u[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      u[i] = (uint32_t)from_float<DT == 1>(acc[2 * i]) |
             ((uint32_t)from_float<DT == 1>(acc[2 * i + 1]) << 16);
    o.x = u[0];
    o.y = u[1];
    o.z = u[2];
    o.w = u[3];
    *reinterpret_cast<uint4*>((uint16_t*)p.y + yoff) = o;
  }
}

}  // namespace

fupr_status launch_status(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return FUPR_OK;
  if (tuning_int("debug", 0)) fprintf(stderr, "fupr: %s: %s\n", what, hipGetErrorString(e));
  return FUPR_ERR_LAUNCH;
}

namespace {

// Geometry of a 16-bit convolution as the kernels take it.
Conv16Params geometry16(const fupr_conv_shape& s, fupr_dtype dt, int N, int H, int W) {
  const PackedLayout L = packed_layout(s, dt);
  Conv16Params p{};
  p.H = H; p.W = W;
  p.P = out_extent(H, s.R, s.stride, s.pad);
  p.Q = out_extent(W, s.S, s.stride, s.pad);
  p.PQ = p.P * p.Q;
  p.M = (int)((int64_t)N * p.PQ);
  p.S = s.S; p.stride = s.stride; p.pad = s.pad;
  p.Kp = L.Kp; p.FT = L.Kp / 16; p.cpt = L.Cp / 8; p.nchunk = L.nchunk; p.nsteps = L.nchunk_pad / 4;
  return p;
}

// A 16-bit convolution's arguments as the kernels take them.
Conv16Params params16(const ConvArgs& a) {
  fupr_conv_shape s{a.K, a.C, a.R, a.S, a.stride, a.pad};
  const PackedLayout L = packed_layout(s, a.dt);
  const char* blob = reinterpret_cast<const char*>(a.packed);
  const int64_t M = (int64_t)a.N * a.P * a.Q;
  Conv16Params p{};
  p.x = (const uint16_t*)a.x;
  p.w = (const uint16_t*)(blob + L.weight_offset);
  p.bias = (const float*)blob;
  p.res = (const uint16_t*)a.res;
  p.y = (uint16_t*)a.y;
  p.H = a.H; p.W = a.W; p.xcs = a.xcs;
  p.P = a.P; p.Q = a.Q; p.PQ = a.P * a.Q; p.M = (int)M; p.ycs = a.ycs;
  p.S = a.S; p.stride = a.stride; p.pad = a.pad;
  p.Kp = L.Kp; p.FT = L.Kp / 16; p.cpt = L.Cp / 8; p.nchunk = L.nchunk; p.nsteps = L.nchunk_pad / 4;
  p.rH = a.rH; p.rW = a.rW; p.rcs = a.rcs; p.rss = a.rss; p.roff = a.roff;
  p.relu = a.relu;
  p.x_bytes = (uint32_t)((int64_t)a.N * a.H * a.W * a.xcs * 2);
  p.w_bytes = (uint32_t)((size_t)L.nchunk_pad * L.Kp * 16);
  p.keep = a.keep; p.keep_n = a.K; p.yC = a.yC;
  p.x2 = (const uint16_t*)a.x2;
  if (a.x2) {
    p.x2_bytes = (uint32_t)((int64_t)a.N * a.H2 * a.W2 * a.xcs2 * 2);
    p.split = a.split_c / 8;
    p.H2 = a.H2; p.W2 = a.W2; p.xcs2 = a.xcs2; p.stride2 = a.stride2;
  }
  return p;
}

// Between the two 1 x 1 kernels (measured per layer on the ResNet-50 workloads):
// the pipelined GEMM wins from 512 input channels on and on the small images of
// the last stages; the streaming kernel wins where pixels are many and filters few.
bool prefer_pipe(const Conv16Params& g) {
  // (a stride-2 projection from 256 channels: 32.1 against 35.5 us at 56 x 56, batch 64)
  // (two input tensors, the second a strided block input, from 256 channels on: the streaming
  // kernel would re-read both tensors once per group of 64 filters)
  return conv1x1_pipe_applies(g) &&
         (g.cpt >= 64 || g.M <= 16384 || ((g.stride == 2 || g.x2) && g.cpt >= 32));
}

}  // namespace

const char* conv_kernel_name(const fupr_conv_shape& s, fupr_dtype dt, int N, int H, int W,
                             bool indexed, bool two_inputs) {
  if (dt == FUPR_F32) return "conv32_direct";
  Conv16Params g = geometry16(s, dt, N, H, W);
  if (two_inputs) {   // a marker that is never dereferenced stands for the second tensor
    g.x2 = reinterpret_cast<const uint16_t*>(uintptr_t(16));
    if (prefer_pipe(g)) return conv1x1_pipe_name(g);
    if (conv1x1_stream_applies(g)) return conv1x1_stream_name(g);
    return conv1x1_pipe_applies(g) ? conv1x1_pipe_name(g) : "none";
  }
  // the indexed epilogue needs LDS of its own, which can change the tile: a marker
  // that is never dereferenced stands for the index list
  if (indexed) g.keep = reinterpret_cast<const int32_t*>(uintptr_t(16));
  if (s.R == 3 && conv_patch_applies(g, N)) return conv_patch_name(g, N);
  if (indexed) return conv16_tiled_name(g.FT, g.nsteps, g.M);
  if (s.R == 1 && prefer_pipe(g)) return conv1x1_pipe_name(g);
  if (s.R == 1 && conv1x1_stream_applies(g)) return conv1x1_stream_name(g);
  if (s.R == 1 && conv1x1_pipe_applies(g)) return conv1x1_pipe_name(g);
  return conv16_tiled_name(g.FT, g.nsteps, g.M);
}

fupr_status launch_conv(const ConvArgs& a, void* stream) {
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  fupr_conv_shape s{a.K, a.C, a.R, a.S, a.stride, a.pad};
  const PackedLayout L = packed_layout(s, a.dt);
  const int64_t M = (int64_t)a.N * a.P * a.Q;
  const char* blob = reinterpret_cast<const char*>(a.packed);
  if (a.dt == FUPR_F32) {
    Conv32Params p;
    p.x = (const float*)a.x;
    p.w = (const float*)(blob + L.weight_offset);
    p.bias = (const float*)blob;
    p.res = (const float*)a.res;
    p.y = (float*)a.y;
    p.H = a.H; p.W = a.W; p.xcs = a.xcs; p.Cp = L.Cp;
    p.P = a.P; p.Q = a.Q; p.PQ = a.P * a.Q; p.M = (int)M; p.ycs = a.ycs;
    p.R = a.R; p.S = a.S; p.stride = a.stride; p.pad = a.pad;
    p.Kp = L.Kp; p.KQ = L.Kp / 4;
    p.rH = a.rH; p.rW = a.rW; p.rcs = a.rcs; p.rss = a.rss; p.roff = a.roff;
    p.relu = a.relu;
    const int64_t threads = M * p.KQ;
    hipLaunchKernelGGL(conv32_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, p);
    return launch_status(__func__);
  }
  const Conv16Params p = params16(a);
  if (a.x2) {   // two input tensors: the two 1 x 1 kernels read them
    if (prefer_pipe(p)) return launch_conv1x1_pipe(p, a.N, a.dt == FUPR_BF16, stream);
    if (conv1x1_stream_applies(p)) return launch_conv1x1_stream(p, a.N, a.dt == FUPR_BF16, stream);
    if (conv1x1_pipe_applies(p)) return launch_conv1x1_pipe(p, a.N, a.dt == FUPR_BF16, stream);
    return FUPR_ERR_LIMIT;
  }
  if (a.R == 3 && conv_patch_applies(p, a.N)) return launch_conv_patch(p, a.N, a.dt == FUPR_BF16, stream);
  // the indexed epilogue exists in the 3 x 3 kernel above and in the general one
  if (a.keep) return launch_conv16_tiled(p, a.dt == FUPR_BF16, stream);
  if (a.R == 1 && prefer_pipe(p)) return launch_conv1x1_pipe(p, a.N, a.dt == FUPR_BF16, stream);
  if (a.R == 1 && conv1x1_stream_applies(p)) return launch_conv1x1_stream(p, a.N, a.dt == FUPR_BF16, stream);
  if (a.R == 1 && conv1x1_pipe_applies(p)) return launch_conv1x1_pipe(p, a.N, a.dt == FUPR_BF16, stream);
  return launch_conv16_tiled(p, a.dt == FUPR_BF16, stream);
}

}  // namespace fupr

// ------------------------------------------------------------------ C ABI ----

using namespace fupr;

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Geometry rules shared by every tensor argument.
fupr_status check_tensor(const fupr_tensor* t) {
  if (!t->ptr) return FUPR_ERR_NULL;
  if (!dtype_ok((int)t->dt)) return FUPR_ERR_DTYPE;
  if (t->N <= 0 || t->H <= 0 || t->W <= 0 || t->C <= 0) return FUPR_ERR_SHAPE;
  if (t->c_stride < t->C || t->c_stride % c_align(t->dt) != 0) return FUPR_ERR_ALIGN;
  if (!aligned16(t->ptr)) return FUPR_ERR_ALIGN;
  if ((int64_t)t->N * t->H * t->W * t->c_stride >= (int64_t(1) << 31)) return FUPR_ERR_LIMIT;
  return FUPR_OK;
}

}  // namespace

namespace {

// Validates one fused convolution call and fills the launcher's arguments.
fupr_status check_conv(const fupr_conv_shape* shape, const fupr_tensor* x, const void* packed,
                       const fupr_residual* res, uint32_t epilogue_flags, const fupr_tensor* y,
                       ConvArgs* out, bool wider_y = false) {
  if (!shape || !x || !y || !packed) return FUPR_ERR_NULL;
  if (!shape_ok(shape)) return FUPR_ERR_SHAPE;
  if (epilogue_flags & ~uint32_t(FUPR_FUSE_RELU | FUPR_FUSE_ADD)) return FUPR_ERR_ARG;
  const bool add = (epilogue_flags & FUPR_FUSE_ADD) != 0;
  if (add && !res) return FUPR_ERR_NULL;
  if (!add && res) return FUPR_ERR_ARG;
  fupr_status st = check_tensor(x);
  if (st != FUPR_OK) return st;
  st = check_tensor(y);
  if (st != FUPR_OK) return st;
  if (x->dt != y->dt) return FUPR_ERR_DTYPE;
  if ((reinterpret_cast<uintptr_t>(packed) & 255u) != 0) return FUPR_ERR_ALIGN;
  const int P = out_extent(x->H, shape->R, shape->stride, shape->pad);
  const int Q = out_extent(x->W, shape->S, shape->stride, shape->pad);
  if (x->H + 2 * shape->pad < shape->R || x->W + 2 * shape->pad < shape->S) return FUPR_ERR_SHAPE;
  if (x->C != shape->C || y->C != shape->K || y->N != x->N || y->H != P || y->W != Q)
    return FUPR_ERR_SHAPE;
  const PackedLayout L = packed_layout(*shape, x->dt);
  if (!wider_y && y->c_stride > L.Kp) return FUPR_ERR_ALIGN;
  if (x->ptr == y->ptr) return FUPR_ERR_ARG;

  ConvArgs a{};
  a.x = x->ptr;
  a.packed = packed;
  a.y = y->ptr;
  a.N = x->N; a.H = x->H; a.W = x->W; a.C = x->C; a.xcs = x->c_stride;
  a.P = P; a.Q = Q; a.K = shape->K; a.ycs = y->c_stride;
  a.R = shape->R; a.S = shape->S; a.stride = shape->stride; a.pad = shape->pad;
  a.relu = (epilogue_flags & FUPR_FUSE_RELU) ? 1 : 0;
  a.dt = x->dt;
  if (add) {
    const fupr_tensor* t = &res->t;
    st = check_tensor(t);
    if (st != FUPR_OK) return st;
    if (t->dt != x->dt) return FUPR_ERR_DTYPE;
    if (res->spatial_stride < 1 || res->c_offset < 0 || res->c_offset % 4 != 0) return FUPR_ERR_ARG;
    if (t->N != x->N || res->c_offset + t->C > shape->K) return FUPR_ERR_SHAPE;
    if ((int64_t)(P - 1) * res->spatial_stride >= t->H ||
        (int64_t)(Q - 1) * res->spatial_stride >= t->W)
      return FUPR_ERR_SHAPE;
    if (t->ptr == y->ptr && !(res->spatial_stride == 1 && res->c_offset == 0 && t->H == P &&
                              t->W == Q && t->c_stride == y->c_stride))
      return FUPR_ERR_ARG;
    a.res = t->ptr;
    a.rH = t->H; a.rW = t->W; a.rC = t->C; a.rcs = t->c_stride;
    a.rss = res->spatial_stride; a.roff = res->c_offset;
  }
  *out = a;
  return FUPR_OK;
}

}  // namespace

extern "C" fupr_status fupr_conv_fused(const fupr_conv_shape* shape, const fupr_tensor* x,
                                       const void* packed, const fupr_residual* res,
                                       uint32_t epilogue_flags, const fupr_tensor* y,
                                       void* stream) {
  ConvArgs a;
  const fupr_status st = check_conv(shape, x, packed, res, epilogue_flags, y, &a);
  return st != FUPR_OK ? st : launch_conv(a, stream);
}

namespace {

// Validates a convolution over two concatenated tensors: x1 as an ordinary 1 x 1
// convolution of its own channels, then x2 and the split.
fupr_status check_conv_cat(const fupr_conv_shape* shape, const fupr_tensor* x1, const fupr_tensor* x2,
                           int32_t x2_stride, const void* packed, const fupr_residual* res,
                           uint32_t epilogue_flags, const fupr_tensor* y, ConvArgs* out) {
  if (!shape || !x1 || !x2) return FUPR_ERR_NULL;
  if (!shape_ok(shape)) return FUPR_ERR_SHAPE;
  if (shape->R != 1 || shape->S != 1 || shape->stride != 1 || shape->pad != 0) return FUPR_ERR_SHAPE;
  if (x2_stride != 1 && x2_stride != 2) return FUPR_ERR_ARG;
  fupr_conv_shape own = *shape;   // the part that reads x1
  own.C = x1->C;
  ConvArgs a;
  fupr_status st = check_conv(&own, x1, packed, res, epilogue_flags, y, &a);
  if (st != FUPR_OK) return st;
  st = check_tensor(x2);
  if (st != FUPR_OK) return st;
  if (x1->dt == FUPR_F32) return FUPR_ERR_DTYPE;
  if (x2->dt != x1->dt) return FUPR_ERR_DTYPE;
  const int split = round_up(x1->C, FUPR_CAT_ALIGN);
  if (shape->C != split + x2->C || x2->N != x1->N) return FUPR_ERR_SHAPE;
  if ((int64_t)(a.P - 1) * x2_stride >= x2->H || (int64_t)(a.Q - 1) * x2_stride >= x2->W)
    return FUPR_ERR_SHAPE;
  if (x2->ptr == y->ptr) return FUPR_ERR_ARG;
  a.C = shape->C;
  a.x2 = x2->ptr;
  a.H2 = x2->H; a.W2 = x2->W; a.xcs2 = x2->c_stride; a.stride2 = x2_stride;
  a.split_c = split;
  *out = a;
  return FUPR_OK;
}

}  // namespace

extern "C" fupr_status fupr_conv_cat_fused(const fupr_conv_shape* shape, const fupr_tensor* x1,
                                           const fupr_tensor* x2, int32_t x2_spatial_stride,
                                           const void* packed, const fupr_residual* res,
                                           uint32_t epilogue_flags, const fupr_tensor* y,
                                           void* stream) {
  ConvArgs a;
  const fupr_status st =
      check_conv_cat(shape, x1, x2, x2_spatial_stride, packed, res, epilogue_flags, y, &a);
  return st != FUPR_OK ? st : launch_conv(a, stream);
}

extern "C" fupr_status fupr_conv_scatter_fused(const fupr_conv_shape* shape, const fupr_tensor* x,
                                               const void* packed, const int32_t* keep_idx,
                                               uint32_t epilogue_flags, const fupr_tensor* y,
                                               void* stream) {
  if (!shape || !x || !y || !packed || !keep_idx) return FUPR_ERR_NULL;
  if (epilogue_flags & ~uint32_t(FUPR_FUSE_RELU)) return FUPR_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(keep_idx) & 3u) != 0) return FUPR_ERR_ALIGN;
  // the convolution's own output has shape->K channels; y is wider
  fupr_tensor own = *y;
  own.C = shape->K;
  if (shape_ok(shape) && shape->K > y->C) return FUPR_ERR_SHAPE;
  ConvArgs a;
  const fupr_status st = check_conv(shape, x, packed, nullptr, epilogue_flags, &own, &a, true);
  if (st != FUPR_OK) return st;
  if (y->C <= 0 || y->c_stride < y->C) return FUPR_ERR_SHAPE;
  if (a.dt == FUPR_F32) return FUPR_ERR_DTYPE;
  a.keep = keep_idx;
  a.yC = y->C;
  return launch_conv(a, stream);
}

extern "C" fupr_status fupr_conv_conv1x1_fused(const fupr_conv_shape* shape1, const fupr_tensor* x,
                                               const void* packed1, const fupr_residual* res,
                                               uint32_t flags1, const fupr_tensor* y,
                                               const fupr_conv_shape* shape2, const void* packed2,
                                               uint32_t flags2, const fupr_tensor* h,
                                               void* stream) {
  ConvArgs a, b;
  fupr_status st = check_conv(shape1, x, packed1, res, flags1, y, &a);
  if (st != FUPR_OK) return st;
  st = check_conv(shape2, y, packed2, nullptr, flags2, h, &b);
  if (st != FUPR_OK) return st;
  if (h->ptr == x->ptr || (res && h->ptr == res->t.ptr)) return FUPR_ERR_ARG;
  if (a.dt == FUPR_F32) return FUPR_ERR_LIMIT;
  const Conv16Params p1 = params16(a), p2 = params16(b);
  if (!conv1x1_fused_pair_applies(p1, p2)) return FUPR_ERR_LIMIT;
  return launch_conv1x1_fused_pair(p1, p2, a.N, a.dt == FUPR_BF16, stream);
}

fupr_status fupr::conv_cat_conv1x1_fused(const fupr_conv_shape* shape1, const fupr_tensor* x1,
                                         const fupr_tensor* x2, int32_t x2_stride,
                                         const void* packed1, uint32_t flags1, const fupr_tensor* y,
                                         const fupr_conv_shape* shape2, const void* packed2,
                                         uint32_t flags2, const fupr_tensor* h, void* stream) {
  ConvArgs a, b;
  fupr_status st = check_conv_cat(shape1, x1, x2, x2_stride, packed1, nullptr, flags1, y, &a);
  if (st != FUPR_OK) return st;
  st = check_conv(shape2, y, packed2, nullptr, flags2, h, &b);
  if (st != FUPR_OK) return st;
  if (h->ptr == x1->ptr || h->ptr == x2->ptr) return FUPR_ERR_ARG;
  const Conv16Params p1 = params16(a), p2 = params16(b);
  if (!conv1x1_fused_pair_applies(p1, p2)) return FUPR_ERR_LIMIT;
  return launch_conv1x1_fused_pair(p1, p2, a.N, a.dt == FUPR_BF16, stream);
}

bool fupr::conv_pair_fusable(const fupr_conv_shape& s1, const fupr_conv_shape& s2, fupr_dtype dt,
                             int N, int H, int W) {
  if (dt == FUPR_F32) return false;
  Conv16Params g1 = geometry16(s1, dt, N, H, W);
  g1.ycs = min_c_stride(s1.K, dt);
  const Conv16Params g2 = geometry16(s2, dt, N, g1.P, g1.Q);
  return s1.R == 1 && s2.R == 1 && conv1x1_fused_pair_applies(g1, g2);
}

extern "C" fupr_status fupr_conv_maxpool_fused(const fupr_conv_shape* shape, const fupr_tensor* x,
                                               const void* packed, int32_t pool_k,
                                               int32_t pool_stride, int32_t pool_pad,
                                               const fupr_tensor* y, void* stream) {
  if (!shape || !x || !y || !packed) return FUPR_ERR_NULL;
  if (!shape_ok(shape)) return FUPR_ERR_SHAPE;
  fupr_status st = check_tensor(x);
  if (st != FUPR_OK) return st;
  st = check_tensor(y);
  if (st != FUPR_OK) return st;
  if (x->dt != y->dt) return FUPR_ERR_DTYPE;
  if ((reinterpret_cast<uintptr_t>(packed) & 255u) != 0) return FUPR_ERR_ALIGN;
  if (pool_k <= 0 || pool_stride <= 0 || pool_pad < 0 || pool_pad >= pool_k) return FUPR_ERR_ARG;
  if (x->H + 2 * shape->pad < shape->R || x->W + 2 * shape->pad < shape->S) return FUPR_ERR_SHAPE;
  const int SH = out_extent(x->H, shape->R, shape->stride, shape->pad);
  const int SW = out_extent(x->W, shape->S, shape->stride, shape->pad);
  if (SH + 2 * pool_pad < pool_k || SW + 2 * pool_pad < pool_k) return FUPR_ERR_SHAPE;
  const int P = out_extent(SH, pool_k, pool_stride, pool_pad);
  const int Q = out_extent(SW, pool_k, pool_stride, pool_pad);
  if (x->C != shape->C || y->C != shape->K || y->N != x->N || y->H != P || y->W != Q)
    return FUPR_ERR_SHAPE;
  if (x->ptr == y->ptr) return FUPR_ERR_ARG;
  if (!stem_pool_applies(*shape, x->dt, x->N, x->H, x->W, x->c_stride, y->c_stride, pool_k,
                         pool_stride, pool_pad))
    return FUPR_ERR_LIMIT;
  return launch_stem_pool(*shape, x->dt, x->N, x->H, x->W, x->c_stride, y->c_stride, x->ptr, packed,
                          y->ptr, stream);
}

namespace {

fupr_status pool_common(const fupr_tensor* x, const fupr_tensor* y) {
  if (!x || !y) return FUPR_ERR_NULL;
  fupr_status st = check_tensor(x);
  if (st != FUPR_OK) return st;
  st = check_tensor(y);
  if (st != FUPR_OK) return st;
  if (x->dt != y->dt) return FUPR_ERR_DTYPE;
  if (x->C != y->C || x->N != y->N) return FUPR_ERR_SHAPE;
  if (y->c_stride > x->c_stride) return FUPR_ERR_ALIGN;
  if (x->ptr == y->ptr) return FUPR_ERR_ARG;
  return FUPR_OK;
}

}  // namespace

extern "C" fupr_status fupr_maxpool(const fupr_tensor* x, int32_t k, int32_t stride, int32_t pad,
                                    const fupr_tensor* y, void* stream) {
  fupr_status st = pool_common(x, y);
  if (st != FUPR_OK) return st;
  if (k <= 0 || stride <= 0 || pad < 0 || pad >= k) return FUPR_ERR_ARG;
  if (x->H + 2 * pad < k || x->W + 2 * pad < k) return FUPR_ERR_SHAPE;
  const int P = out_extent(x->H, k, stride, pad), Q = out_extent(x->W, k, stride, pad);
  if (y->H != P || y->W != Q) return FUPR_ERR_SHAPE;
  // every window must hold at least one tap inside the image
  if ((int64_t)(P - 1) * stride - pad >= x->H || (int64_t)(Q - 1) * stride - pad >= x->W)
    return FUPR_ERR_SHAPE;
  PoolParams p;
  p.x = x->ptr; p.y = y->ptr;
  p.H = x->H; p.W = x->W; p.cs = x->c_stride; p.P = P; p.Q = Q; p.ycs = y->c_stride;
  p.k = k; p.stride = stride; p.pad = pad;
  p.chunks = y->c_stride / c_align(x->dt);
  p.total = (int64_t)x->N * P * Q * p.chunks;
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  dim3 grid((unsigned)((p.total + 255) / 256));
  if (x->dt == FUPR_F32) hipLaunchKernelGGL(maxpool_kernel<0>, grid, dim3(256), 0, hs, p);
  else if (x->dt == FUPR_BF16) hipLaunchKernelGGL(maxpool_kernel<1>, grid, dim3(256), 0, hs, p);
  else hipLaunchKernelGGL(maxpool_kernel<2>, grid, dim3(256), 0, hs, p);
  return launch_status(__func__);
}

extern "C" fupr_status fupr_global_avgpool(const fupr_tensor* x, const fupr_tensor* y,
                                           void* stream) {
  fupr_status st = pool_common(x, y);
  if (st != FUPR_OK) return st;
  if (y->H != 1 || y->W != 1) return FUPR_ERR_SHAPE;
  PoolParams p{};
  p.x = x->ptr; p.y = y->ptr;
  p.H = x->H; p.W = x->W; p.cs = x->c_stride; p.P = 1; p.Q = 1; p.ycs = y->c_stride;
  p.chunks = y->c_stride / c_align(x->dt);
  p.total = (int64_t)x->N * p.chunks;
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  dim3 grid((unsigned)((p.total + 31) / 32));
  if (x->dt == FUPR_F32) hipLaunchKernelGGL(avgpool_kernel<0>, grid, dim3(256), 0, hs, p);
  else if (x->dt == FUPR_BF16) hipLaunchKernelGGL(avgpool_kernel<1>, grid, dim3(256), 0, hs, p);
  else hipLaunchKernelGGL(avgpool_kernel<2>, grid, dim3(256), 0, hs, p);
  return launch_status(__func__);
}
