// The ImageNet stem of Table II in one kernel: 7 x 7 stride-2 convolution of a
// 3-channel image (bias and ReLU in the epilogue, Sec. VI-B-3) followed by the
// 3 x 3 stride-2 max-pool.  The convolution's output, the largest tensor of
// the network, never reaches memory: a workgroup computes the (2 TP + 1) x
// (2 TQ + 1) convolution outputs that a TP x TQ tile of pool outputs needs,
// keeps them in LDS, and stores only the maxima.
//
// GEMM view: rows = 64 filters (MFMA operand A), columns = convolution pixels
// (operand B).  The reduction index is (r, column pair j, 2 pixels x 4 channels):
// with 4 channels per pixel in LDS (the fourth is zero) the 8 values one lane
// feeds an MFMA with are two neighbouring input pixels = 16 contiguous bytes,
// so the 7 x 7 x 3 = 147 products per output take 7 MFMA 16x16x32 steps
// (7 rows x 4 pairs x 8 = 224, tap s = 7 and channel 3 have zero weights)
// instead of the 13 steps of one 8-channel chunk per tap.  The filter fragments
// are rebuilt from the packed blob once per workgroup and stay in registers.
//
// Max-pool over ReLU outputs: positions outside the convolution's output count
// as 0, which never wins against the window's centre tap (>= 0, always inside).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <mutex>

#include "device_utils.h"
#include "fupr.h"
#include "layout.h"
#include "stem_pool.h"

namespace fupr {
namespace {

constexpr uint32_t kOutside = 0x80000000u;
constexpr int kMaxStemPatchLoads = 8;  // 8-byte pixels of the input patch per thread
constexpr int kStemPixelBytes = 144;   // 64 channels + 16 bytes: spreads LDS banks

struct StemParams {
  const uint16_t* x;
  const uint16_t* w;     // [49 (+3)][64][8]
  const float* bias;
  uint16_t* y;
  uint32_t x_bytes, w_bytes;
  int H, W, xcs;         // input
  int SH, SW;            // convolution output
  int P, Q, ycs;         // pool output
  int TP, TQ;            // pool outputs per workgroup
  int tiles_p, tiles_q;  // per image
  int total_tiles;
  int th, tw;            // convolution outputs per workgroup: 2 TP + 1, 2 TQ + 1
  int PH, PW;            // input patch: 2 th + 5 rows, 2 tw + 5 columns rounded up to even
  int n_ctiles;          // 16-pixel tiles of th * tw
  int patch_off, stem_off;   // LDS byte offsets (the filter staging area starts at 0)
  FastDiv div_tw, div_PW, div_TQ, div_image, div_tq;   // by tw, PW, TQ, tiles per image, tiles_q
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short short8_t __attribute__((ext_vector_type(8)));

template <bool BF>
__global__ __launch_bounds__(256) void stem_pool_kernel(const StemParams p) {
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, g = lane >> 4;

  const int per_image = p.tiles_p * p.tiles_q;
  const __amdgpu_buffer_rsrc_t xrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x), 0, p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t wrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.w), 0, p.w_bytes, 0x00020000);

  // ---- filters: [r * 4 + j][filter][2 taps x 4 channels] in LDS, then registers -----
  for (int e = tid; e < 28 * 64; e += 256) {
    const int ch = e >> 6, f = e & 63;
    const int r = ch >> 2, j = ch & 3;
    const int tap = r * 7 + 2 * j;
    const u32x2 lo = __builtin_amdgcn_raw_buffer_load_b64(wrsrc, (uint32_t)(tap * 64 + f) * 16u, 0, 0);
    const u32x2 hi = __builtin_amdgcn_raw_buffer_load_b64(
        wrsrc, 2 * j + 1 < 7 ? (uint32_t)((tap + 1) * 64 + f) * 16u : kOutside, 0, 0);
    *reinterpret_cast<uint4*>(lds + e * 16) = uint4{lo[0], lo[1], hi[0], hi[1]};
  }
  f32x4 bias4[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) bias4[t] = *reinterpret_cast<const f32x4*>(p.bias + t * 16 + g * 4);
  __syncthreads();
  uint4 a[7][4];
#pragma unroll
  for (int k = 0; k < 7; ++k)
#pragma unroll
    for (int t = 0; t < 4; ++t)
      a[k][t] = *reinterpret_cast<const uint4*>(lds + (((k * 4 + g) * 64) + t * 16 + li) * 16);
  // (the first barrier of the tile loop frees the staging area for the convolution tile)

  char* patch = lds + p.patch_off;
  char* stem = lds + p.stem_off;
  const int n_cpix = p.th * p.tw;
  const int prow_bytes = p.PW * 8;
  const int ychunks = p.ycs >> 3;
  const int n_patch = p.PH * p.PW;

  // the input patch of a tile: [PH][PW][4 channels], fetched one tile ahead
  u32x2 pre[kMaxStemPatchLoads];
  int slot_rc[kMaxStemPatchLoads];   // patch row << 16 | patch column of this thread's pixels
#pragma unroll
  for (int i = 0; i < kMaxStemPatchLoads; ++i) {
    const int e = tid + i * 256;
    const int pr = div_by(e, p.div_PW), pc = e - pr * p.PW;
    slot_rc[i] = e < n_patch ? (pr << 16 | pc) : -1;
  }
  auto fetch = [&](int tile) {
    const int n = div_by(tile, p.div_image), rem = tile - n * per_image;
    const int tp = div_by(rem, p.div_tq), tq = rem - tp * p.tiles_q;
    const int h0 = 4 * tp * p.TP - 5, w0 = 4 * tq * p.TQ - 5;   // first input pixel
#pragma unroll
    for (int i = 0; i < kMaxStemPatchLoads; ++i) {
      const int ih = h0 + (slot_rc[i] >> 16), iw = w0 + (slot_rc[i] & 0xffff);
      const bool ok = slot_rc[i] >= 0 && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
      const uint32_t off = ok ? (uint32_t)(((n * p.H + ih) * p.W + iw) * p.xcs) * 2u : kOutside;
      pre[i] = __builtin_amdgcn_raw_buffer_load_b64(xrsrc, off, 0, 0);
    }
  };

  int tile = blockIdx.x;
  if (tile < p.total_tiles) fetch(tile);
  for (; tile < p.total_tiles; tile += gridDim.x) {
    const int n = div_by(tile, p.div_image), rem = tile - n * per_image;
    const int tp = div_by(rem, p.div_tq), tq = rem - tp * p.tiles_q;
    const int p0 = tp * p.TP, q0 = tq * p.TQ;      // first pool output
    const int a0 = 2 * p0 - 1, b0 = 2 * q0 - 1;    // first convolution output
#pragma unroll
    for (int i = 0; i < kMaxStemPatchLoads; ++i) {
      const int e = tid + i * 256;
      if (slot_rc[i] >= 0) *reinterpret_cast<u32x2*>(patch + e * 8) = pre[i];
    }
    __syncthreads();   // patch complete; the previous tile's maxima have been taken
    if (tile + (int)gridDim.x < p.total_tiles) fetch(tile + gridDim.x);

    // ---- convolution tile -> LDS ---------------------------------------------------
    for (int ct = wave; ct < p.n_ctiles; ct += 4) {
      const int cp = ct * 16 + li;
      const int cpc = min(cp, n_cpix - 1);
      const int sr = div_by(cpc, p.div_tw), sc = cpc - sr * p.tw;
      const char* bp = patch + (2 * sr * p.PW + 2 * sc) * 8 + g * 16;
      uint4 b[7];
#pragma unroll
      for (int k = 0; k < 7; ++k) b[k] = *reinterpret_cast<const uint4*>(bp + k * prow_bytes);
      f32x4 acc[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) acc[t] = bias4[t];
#pragma unroll
      for (int k = 0; k < 7; ++k)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = mfma_16x16x32<BF>(a[k][t], b[k], acc[t]);
      const int sh = a0 + sr, sw = b0 + sc;
      const bool inside = sh >= 0 && sh < p.SH && sw >= 0 && sw < p.SW;
      if (cp < n_cpix) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          u32x2 o;
          o[0] = inside ? pack2<BF>(fmaxf(acc[t][0], 0.f), fmaxf(acc[t][1], 0.f)) : 0u;
          o[1] = inside ? pack2<BF>(fmaxf(acc[t][2], 0.f), fmaxf(acc[t][3], 0.f)) : 0u;
          *reinterpret_cast<u32x2*>(stem + cp * kStemPixelBytes + t * 32 + g * 8) = o;
        }
      }
    }
    __syncthreads();   // tile complete; the patch may be overwritten

    // ---- 3 x 3 stride-2 maxima: one thread per (pool pixel, 8 channels) -------------
    // non-negative values of either 16-bit format order like their bit patterns
    for (int e = tid; e < p.TP * p.TQ * 8; e += 256) {
      const int c8 = e & 7, pix = e >> 3;
      const int pp = div_by(pix, p.div_TQ), qq = pix - pp * p.TQ;
      const int gp = p0 + pp, gq = q0 + qq;
      if (gp >= p.P || gq >= p.Q || c8 >= ychunks) continue;
      short8_t m = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) {
          const uint4 v = *reinterpret_cast<const uint4*>(
              stem + ((2 * pp + r) * p.tw + 2 * qq + s) * kStemPixelBytes + c8 * 16);
          m = __builtin_elementwise_max(m, __builtin_bit_cast(short8_t, v));
        }
      *reinterpret_cast<uint4*>(p.y + (((size_t)n * p.P + gp) * p.Q + gq) * p.ycs + c8 * 8) =
          __builtin_bit_cast(uint4, m);
    }
  }
}

int stem_compute_units() {
  static int cus = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        n <= 0) {
      (void)hipGetLastError();
      return 256;
    }
    return n;
  }();
  return cus;
}

bool plan_stem(const fupr_conv_shape& s, fupr_dtype dt, int N, int H, int W, int xcs, int ycs,
               int pool_k, int pool_stride, int pool_pad, StemParams* out, size_t* lds_bytes,
               int64_t* grid) {
  if (dt != FUPR_BF16 && dt != FUPR_F16) return false;
  if (s.R != 7 || s.S != 7 || s.stride != 2 || s.pad != 3 || s.C > 4 || s.K != 64) return false;
  if (pool_k != 3 || pool_stride != 2 || pool_pad != 1) return false;
  if (xcs % 4 != 0 || ycs != 64) return false;
  StemParams p{};
  p.H = H; p.W = W; p.xcs = xcs;
  p.SH = out_extent(H, 7, 2, 3);
  p.SW = out_extent(W, 7, 2, 3);
  p.P = out_extent(p.SH, 3, 2, 1);
  p.Q = out_extent(p.SW, 3, 2, 1);
  p.ycs = ycs;
  // 8 x 7 pool outputs need 17 x 15 = 255 convolution outputs: 16 full MFMA tiles
  p.TP = std::min(8, p.P);
  p.TQ = std::min(7, p.Q);
  p.tiles_p = (p.P + p.TP - 1) / p.TP;
  p.tiles_q = (p.Q + p.TQ - 1) / p.TQ;
  p.th = 2 * p.TP + 1;
  p.tw = 2 * p.TQ + 1;
  p.PH = 2 * p.th + 5;
  p.PW = (2 * p.tw + 5 + 1) & ~1;
  p.n_ctiles = (p.th * p.tw + 15) / 16;
  const int stage_bytes = 28 * 64 * 16;
  const int stem_bytes = p.th * p.tw * kStemPixelBytes;
  p.stem_off = 0;   // over the staging area, which is dead by then
  p.patch_off = round_up(std::max(stage_bytes, stem_bytes), 16);
  *lds_bytes = (size_t)p.patch_off + (size_t)p.PH * p.PW * 8;
  if (*lds_bytes > 64 * 1024) return false;
  p.div_tw = fast_div(p.tw);
  p.div_PW = fast_div(p.PW);
  p.div_TQ = fast_div(p.TQ);
  p.div_image = fast_div(p.tiles_p * p.tiles_q);
  p.div_tq = fast_div(p.tiles_q);
  if (p.PH * p.PW > kMaxStemPatchLoads * 256 || p.th * p.tw + 16 >= 65536) return false;
  if ((int64_t)N * H * W * xcs * 2 >= (int64_t)kOutside) return false;
  const int64_t total = (int64_t)N * p.tiles_p * p.tiles_q;
  if (total >= (int64_t(1) << 30)) return false;
  p.total_tiles = (int)total;
  *grid = std::min<int64_t>(total, 2 * (int64_t)stem_compute_units());   // two workgroups fit a compute unit
  *out = p;
  return true;
}

}  // namespace

bool stem_pool_applies(const fupr_conv_shape& s, fupr_dtype dt, int N, int H, int W, int xcs,
                       int ycs, int pool_k, int pool_stride, int pool_pad) {
  StemParams p;
  size_t lds;
  int64_t grid;
  return plan_stem(s, dt, N, H, W, xcs, ycs, pool_k, pool_stride, pool_pad, &p, &lds, &grid);
}

fupr_status launch_stem_pool(const fupr_conv_shape& s, fupr_dtype dt, int N, int H, int W, int xcs,
                             int ycs, const void* x, const void* packed, void* y, void* stream) {
  StemParams p;
  size_t lds;
  int64_t grid;
  if (!plan_stem(s, dt, N, H, W, xcs, ycs, 3, 2, 1, &p, &lds, &grid)) return FUPR_ERR_LIMIT;
  const PackedLayout L = packed_layout(s, dt);
  const char* blob = reinterpret_cast<const char*>(packed);
  p.x = reinterpret_cast<const uint16_t*>(x);
  p.w = reinterpret_cast<const uint16_t*>(blob + L.weight_offset);
  p.bias = reinterpret_cast<const float*>(blob);
  p.y = reinterpret_cast<uint16_t*>(y);
  p.x_bytes = (uint32_t)((int64_t)N * H * W * xcs * 2);
  p.w_bytes = (uint32_t)((size_t)L.nchunk_pad * L.Kp * 16);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  static std::once_flag once;
  static hipError_t status = hipSuccess;
  std::call_once(once, [] {
    status = hipFuncSetAttribute(reinterpret_cast<const void*>(&stem_pool_kernel<true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
    if (status == hipSuccess)
      status = hipFuncSetAttribute(reinterpret_cast<const void*>(&stem_pool_kernel<false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
  });
  if (status != hipSuccess) return FUPR_ERR_LAUNCH;
  if (dt == FUPR_BF16)
    hipLaunchKernelGGL(stem_pool_kernel<true>, dim3((unsigned)grid), dim3(256), lds, st, p);
  else
    hipLaunchKernelGGL(stem_pool_kernel<false>, dim3((unsigned)grid), dim3(256), lds, st, p);
  return launch_status("stem_pool_kernel");
}

}  // namespace fupr
