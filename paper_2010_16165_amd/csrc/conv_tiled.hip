// 16-bit implicit-GEMM convolution with LDS-staged filters and register-blocked
// tiles: the per-layer kernel for the convolution operator k x c x r x s
// (Sec. III; Sec. IV-B-1 of the paper) at the channel counts filter removal
// leaves (Alg. 1).
//
// GEMM view: rows = filters (MFMA operand A), columns =
// output pixels (operand B), reduction over (r, s, c) in chunks of 8 channels,
// 4 chunks per MFMA 16x16x32 step; the chunk order, and therefore the order of
// every fp32 accumulation, is the same in all conv kernels of this library.
//
// A workgroup of 4 waves (WM x WN) computes WM*MT*16 pixels x WN*NT*16 filters.
//   - Filters: KS steps at a time are copied global -> registers -> LDS, double
//     buffered, one barrier per KS steps; the copy of stage s+1 is in flight
//     while stage s is multiplied.  Every wave reads its NT fragments per step
//     from LDS.
//   - Pixels: each lane loads its own 16 bytes (8 channels of one tap of one
//     pixel) straight from global memory KS steps ahead of use; a tap outside
//     the image contributes zeros.  The 3x3 re-reads hit L1/L2.
//   - Workgroups are numbered so that each XCD (its own L2) works on a
//     contiguous range of pixel blocks and all filter groups of those blocks.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>

#include "conv16.h"
#include "device_utils.h"
#include "layout.h"
#include "tuning.h"

namespace fupr {
namespace {

template <bool BF, int MT, int NT, int WM, int WN, int KS>
__global__ __launch_bounds__(256) void conv16_tiled_kernel(const Conv16Params p, int fgroups,
                                                           int units, int per_xcd) {
  constexpr int BNF = WN * NT * 16;        // filters per workgroup
  constexpr int BMPX = WM * MT * 16;       // pixels per workgroup
  constexpr int STAGE = KS * 4 * BNF;      // uint4 per filter stage
  constexpr int CP = (STAGE + 255) / 256;  // uint4 per thread per stage

  extern __shared__ uint4 smem[];
  uint4* wlds = smem;                                         // [2][STAGE]
  int2* tap_table = reinterpret_cast<int2*>(smem + 2 * STAGE);  // [nsteps * 4]

  // XCD-aware numbering: hardware deals consecutive workgroups round-robin to 8 XCDs
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int unit = xcd * per_xcd + local;
  if (local >= per_xcd || unit >= units) return;
  const int pb = unit / fgroups, fgi = unit - pb * fgroups;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, g = lane >> 4;
  const int wm = wave % WM, wn = wave / WM;
  const int f0 = fgi * BNF;                // first filter of the workgroup
  const int nchunk_pad = p.nsteps * 4;
  // Buffer descriptors: a load whose offset lies outside the tensor returns
  // zeros, so neither the pixel loads nor the filter loads need a branch (a load
  // under a branch would force every wait to drain all loads in flight).
  const __amdgpu_buffer_rsrc_t xrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x), 0, p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t wrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.w), 0, p.w_bytes, 0x00020000);
  constexpr uint32_t kOutside = 0xfffffff0u;

  uint4 wreg[CP];
  auto stage_fetch = [&](int stage) {
#pragma unroll
    for (int k = 0; k < CP; ++k) {
      const int i = tid + k * 256;
      const int cl = i / BNF, f = i - cl * BNF;
      const int chunk = stage * (KS * 4) + cl, gf = f0 + f;
      const bool ok = i < STAGE && gf < p.Kp;   // chunks past the end are outside the buffer
      const uint32_t off = ok ? (uint32_t)(chunk * p.Kp + gf) * 16u : kOutside;
      wreg[k] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(wrsrc, off, 0, 0));
    }
  };
  auto stage_commit = [&](int buf) {
#pragma unroll
    for (int k = 0; k < CP; ++k) {
      const int i = tid + k * 256;
      if (i < STAGE) wlds[buf * STAGE + i] = wreg[k];
    }
  };

  stage_fetch(0);
  for (int j = tid; j < nchunk_pad; j += 256) {
    int2 e;
    if (j < p.nchunk) {
      const int tap = j / p.cpt, c8 = j - tap * p.cpt;
      const int r = tap / p.S, s = tap - r * p.S;
      e.x = ((r * p.W + s) * p.xcs + c8 * 8) * 2;   // bytes
      e.y = (r << 8) | s;
    } else {
      e.x = 0;
      e.y = -1;
    }
    tap_table[j] = e;
  }

  int ih0[MT], iw0[MT];
  uint32_t xoff[MT];   // byte offset of the window's first pixel, modulo 2^32
  bool pv[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = pb * BMPX + (wm * MT + mt) * 16 + li;
    pv[mt] = m < p.M;
    const int mm = pv[mt] ? m : 0;
    const int n = mm / p.PQ, rem = mm - n * p.PQ;
    const int pp = rem / p.Q, qq = rem - pp * p.Q;
    ih0[mt] = pp * p.stride - p.pad;
    iw0[mt] = qq * p.stride - p.pad;
    xoff[mt] = (uint32_t)((n * p.H + ih0[mt]) * p.W + iw0[mt]) * (uint32_t)(p.xcs * 2);
  }

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  stage_commit(0);
  __syncthreads();   // tap table and filter stage 0 are visible

  // Pixel operands of one stage, in registers: bc is multiplied while bn is in flight.
  uint4 bc[KS][MT], bn[KS][MT];
  auto fetch_pixels = [&](int stage) {
#pragma unroll
    for (int d = 0; d < KS; ++d) {
      const int step = min(stage * KS + d, p.nsteps - 1);
      const int2 e = tap_table[step * 4 + g];
      const int r = e.y >> 8, s = e.y & 255;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const bool ok = pv[mt] && e.y >= 0 && (unsigned)(ih0[mt] + r) < (unsigned)p.H &&
                        (unsigned)(iw0[mt] + s) < (unsigned)p.W;
        const uint32_t off = ok ? xoff[mt] + (uint32_t)e.x : kOutside;
        bn[d][mt] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off, 0, 0));
      }
    }
  };
  auto rotate_pixels = [&]() {
#pragma unroll
    for (int d = 0; d < KS; ++d)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) bc[d][mt] = bn[d][mt];
  };
  fetch_pixels(0);
  rotate_pixels();

  // All global loads of stage st+1 are issued before stage st is multiplied and
  // are first touched after it, so the only wait for memory sits at the stage end.
  const int nstages = (p.nsteps + KS - 1) / KS;
  for (int st = 0; st < nstages; ++st) {
    const bool more = st + 1 < nstages;
    if (more) {
      stage_fetch(st + 1);
      fetch_pixels(st + 1);
    }
    const uint4* wl = wlds + (st & 1) * STAGE + g * BNF + wn * NT * 16 + li;
#pragma unroll
    for (int d = 0; d < KS; ++d) {
      if (st * KS + d < p.nsteps) {
        uint4 a[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) a[t] = wl[d * 4 * BNF + t * 16];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int t = 0; t < NT; ++t) acc[mt][t] = mfma_16x16x32<BF>(a[t], bc[d][mt], acc[mt][t]);
      }
    }
    if (more) {
      stage_commit((st + 1) & 1);
      rotate_pixels();
    }
    __syncthreads();
  }

  if (p.keep) {
    // Pruned output filters of a block: filter k adds into channel keep[k] of y,
    // which holds the shortcut; one rounding, 2-byte accesses.  No branch stands
    // between the loads: a filter that does not exist or points outside y reads
    // channel 0 and stores nothing.
    int ch[NT][4];
    float bs[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int ftile = fgi * (WN * NT) + wn * NT + t;
      const int k0 = ftile * 16 + g * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const bool exists = ftile < p.FT && k0 + i < p.keep_n;
        const int c = p.keep[exists ? k0 + i : 0];
        ch[t][i] = exists && (unsigned)c < (unsigned)p.yC ? c : -1;
        bs[t][i] = p.bias[exists ? k0 + i : 0];
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = pb * BMPX + (wm * MT + mt) * 16 + li;
      uint16_t* yp = p.y + (int64_t)min(m, p.M - 1) * p.ycs;
      uint16_t old[NT][4];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) old[t][i] = yp[max(ch[t][i], 0)];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float v = acc[mt][t][i] + bs[t][i] + to_float<BF>(old[t][i]);
          if (p.relu) v = fmaxf(v, 0.f);
          if (m < p.M && ch[t][i] >= 0) yp[ch[t][i]] = from_float<BF>(v);
        }
    }
    return;
  }

  // Epilogue: bias, shortcut, ReLU, one rounding, 8-byte NHWC store.
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = pb * BMPX + (wm * MT + mt) * 16 + li;
    if (m >= p.M) continue;
    const uint16_t* rp = nullptr;
    if (p.res) {
      const int n = m / p.PQ, rem = m - n * p.PQ;
      const int pp = rem / p.Q, qq = rem - pp * p.Q;
      rp = p.res + (((int64_t)n * p.rH + pp * p.rss) * p.rW + qq * p.rss) * p.rcs;
    }
    uint16_t* yp = p.y + (int64_t)m * p.ycs;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int ftile = fgi * (WN * NT) + wn * NT + t;
      const int k0 = ftile * 16 + g * 4;
      if (ftile >= p.FT || k0 >= p.ycs) continue;
      const float4 b4 = *reinterpret_cast<const float4*>(p.bias + k0);
      float v[4] = {acc[mt][t][0] + b4.x, acc[mt][t][1] + b4.y, acc[mt][t][2] + b4.z,
                    acc[mt][t][3] + b4.w};
      if (rp) {
        const int kk = k0 - p.roff;
        if (kk >= 0 && kk < p.rcs) {
          const uint2 rv = *reinterpret_cast<const uint2*>(rp + kk);
          v[0] += to_float<BF>((uint16_t)(rv.x & 0xffffu));
          v[1] += to_float<BF>((uint16_t)(rv.x >> 16));
          v[2] += to_float<BF>((uint16_t)(rv.y & 0xffffu));
          v[3] += to_float<BF>((uint16_t)(rv.y >> 16));
        }
      }
      if (p.relu) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
      }
      uint2 o;
      o.x = pack2<BF>(v[0], v[1]);
      o.y = pack2<BF>(v[2], v[3]);
      *reinterpret_cast<uint2*>(yp + k0) = o;
    }
  }
}

// ---- tile table -----------------------------------------------------------------

struct TileCfg {
  int MT, NT;
  const char* name;
};

// Every instantiated tile: 4 waves side by side along the pixels, MT pixel
// tiles x NT filter tiles of 16 each per wave.
constexpr TileCfg kTiles[] = {
    {1, 1, "conv16t_64x16"}, {2, 1, "conv16t_128x16"}, {1, 2, "conv16t_64x32"}, {2, 2, "conv16t_128x32"},
    {1, 3, "conv16t_64x48"}, {2, 3, "conv16t_128x48"}, {1, 4, "conv16t_64x64"}, {2, 4, "conv16t_128x64"},
    {1, 6, "conv16t_64x96"}, {2, 6, "conv16t_128x96"}, {1, 8, "conv16t_64x128"}, {2, 8, "conv16t_128x128"},
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
constexpr int kStageSteps = 4;

// The tuning switch conv_tile=<tile name> forces one tile for every layer (an
// aid for tests and sweeps, not needed in normal use).
int forced_tile() {
  char e[64];
  if (!tuning_text("conv_tile", e, sizeof(e))) return -1;
  for (int i = 0; i < kNumTiles; ++i)
    if (strcmp(e, kTiles[i].name) == 0) return i;
  return -1;
}

// Tile of a layer with FT filter tiles and M output pixels.  The rule is the
// one that lost least against the per-layer best in a sweep of all tiles over
// every layer shape of the ResNet-18 and ResNet-50 workloads (the layers are
// bound by memory latency, not MFMA issue, so mid-size tiles with several
// workgroups per compute unit win over the largest ones):
//   filters per workgroup: 16 * nt, nt from {1, 2, 3, 4, 6} with the least padded
//       work, narrow workgroups weighted up (see below), the larger nt on a tie;
//   pixels per workgroup: 128, or 64 when 128 would leave fewer than 128 workgroups.
int choose_tile(int FT, int nsteps, int64_t M) {
  (void)nsteps;
  const int f = forced_tile();
  if (f >= 0) return f;
  // filter tiles per workgroup: least padded work, where a workgroup of 1 (2)
  // filter tiles costs about 1.5 (1.2) times as much per tile as a wider one
  // (each pixel fragment it loads feeds that many fewer MFMAs)
  static const int nts[] = {1, 2, 3, 4, 6};
  static const double cost[] = {1.5, 1.2, 1.0, 1.0, 1.0};
  int nt = 1;
  double best = 1e30;
  for (int i = 0; i < 5; ++i) {
    const int c = nts[i], groups = (FT + c - 1) / c;
    const double score = groups * c * cost[i];
    if (score < best - 1e-9 || (score < best + 1e-9 && c > nt)) {
      best = score;
      nt = c;
    }
  }
  const int64_t groups = (FT + nt - 1) / nt;
  const int mt = ((M + 127) / 128) * groups >= 128 ? 2 : 1;
  for (int i = 0; i < kNumTiles; ++i)
    if (kTiles[i].MT == mt && kTiles[i].NT == nt) return i;
  return 0;
}

template <bool BF, int MT, int NT>
fupr_status launch_tile(const Conv16Params& p, hipStream_t st) {
  constexpr int KS = kStageSteps, WM = 4, WN = 1;
  constexpr int BNF = WN * NT * 16, BMPX = WM * MT * 16;
  const int64_t mblocks = ((int64_t)p.M + BMPX - 1) / BMPX;
  const int fgroups = (p.Kp + BNF - 1) / BNF;
  const int64_t units = mblocks * fgroups;
  if (units >= (int64_t(1) << 30)) return FUPR_ERR_LIMIT;
  const int per_xcd = (int)((units + 7) / 8);
  const size_t shmem = (size_t)2 * KS * 4 * BNF * 16 + (size_t)p.nsteps * 4 * sizeof(int2);
  auto kernel = conv16_tiled_kernel<BF, MT, NT, WM, WN, KS>;
  if (shmem > 64 * 1024) {
    static const hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return FUPR_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)(per_xcd * 8)), dim3(256), shmem, st, p, fgroups,
                     (int)units, per_xcd);
  return launch_status("conv16_tiled_kernel");
}

template <bool BF>
fupr_status dispatch(const Conv16Params& p, int tile, hipStream_t st) {
  switch (tile) {
    case 0: return launch_tile<BF, 1, 1>(p, st);
    case 1: return launch_tile<BF, 2, 1>(p, st);
    case 2: return launch_tile<BF, 1, 2>(p, st);
    case 3: return launch_tile<BF, 2, 2>(p, st);
    case 4: return launch_tile<BF, 1, 3>(p, st);
    case 5: return launch_tile<BF, 2, 3>(p, st);
    case 6: return launch_tile<BF, 1, 4>(p, st);
    case 7: return launch_tile<BF, 2, 4>(p, st);
    case 8: return launch_tile<BF, 1, 6>(p, st);
    case 9: return launch_tile<BF, 2, 6>(p, st);
    case 10: return launch_tile<BF, 1, 8>(p, st);
    default: return launch_tile<BF, 2, 8>(p, st);
  }
}

}  // namespace

const char* conv16_tiled_name(int FT, int nsteps, int64_t M) {
  return kTiles[choose_tile(FT, nsteps, M)].name;
}

fupr_status launch_conv16_tiled(const Conv16Params& p, bool bf16, void* stream) {
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int tile = choose_tile(p.FT, p.nsteps, p.M);
  return bf16 ? dispatch<true>(p, tile, st) : dispatch<false>(p, tile, st);
}

}  // namespace fupr
