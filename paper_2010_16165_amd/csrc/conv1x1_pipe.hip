// 1 x 1 convolution (Sec. III: operator k x c x 1 x 1) as a pipelined GEMM for
// the layers whose filters do not fit in LDS at once: the deep first
// convolutions of the later bottleneck stages (1024 -> 128, 2048 -> 256
// channels), the stride-2 projection shortcuts, the fully-connected layer.
//
// Same skeleton as the 3 x 3 kernel: rows = filters (MFMA operand A), columns =
// output pixels (operand B); a unit is a few steps of 32 channels of one tile of
// BM pixels x NF filters; pixels and weights of the following units go global ->
// LDS through range-checked loads issued by four loading waves while the
// computing waves multiply the current unit; a ring of 3 - 4 buffers keeps 2 - 3
// units in flight (these layers multiply little per byte: memory latency times
// the bytes in flight bounds them); one barrier per unit; workgroups are
// persistent over a contiguous range of tiles, so the loads of the next tile
// fly during the last units of the current one.
// Epilogue: bias, shortcut, ReLU, one rounding, 16-byte accesses (pairs of
// filter tiles exchanged between 16-lane rows).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <mutex>

#include "conv16.h"
#include "device_utils.h"
#include "fupr.h"
#include "layout.h"
#include "tuning.h"

namespace fupr {
namespace {

constexpr uint32_t kOutside = 0x80000000u;
constexpr size_t kPipeLdsLimit = 160 * 1024;
constexpr int kLoaderWaves = 4;

struct PipeParams {
  const uint16_t* x;
  const uint16_t* w;     // [nchunk_pad][Kp][8]
  const float* bias;
  const uint16_t* res;
  uint16_t* y;
  uint32_t x_bytes, w_bytes, y_bytes, res_bytes;
  int H, W, xcs;
  int P, Q, PQ, M, ycs;
  int stride;
  int Kp, cpt, n_units;  // units per tile: ceil(cpt / (4 * steps per unit))
  int rH, rW, rcs, rss, roff;
  int relu;
  int plain;             // output pixel m is input pixel m and shortcut pixel m
  int fgroups, tiles;
  int tiles_q, tiles_r;  // tiles / grid, tiles % grid
  FastDiv divPQ, divQ, divF;
  // second input tensor: chunks from `split` on come from x2 at spatial stride
  // stride2 (split is a multiple of 4; 1 << 30 when there is no second tensor)
  const uint16_t* x2;
  uint32_t x2_bytes;
  int split, H2, W2, xcs2, stride2;
};

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short short2_t __attribute__((ext_vector_type(2)));
typedef void __attribute__((address_space(3)))* LdsPtr;

// lane i moves the 16 bytes at offset off of the buffer to the i-th slot after
// lds_base; an offset outside the buffer writes zeros
__device__ __forceinline__ void pipe_load_to_lds(const i32x4& rsrc, uint32_t off,
                                                 uint32_t lds_base) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "buffer_load_dwordx4 %1, %2, 0 offen lds"
      :
      : "s"(lds_base), "v"(off), "s"(rsrc)
      : "memory", "m0");
}

__device__ __forceinline__ i32x4 pipe_rsrc(const void* base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}

__device__ __forceinline__ uint32_t pipe_clamp(uint32_t v, uint32_t floor2) {
  const short2_t a = __builtin_bit_cast(short2_t, v), f = __builtin_bit_cast(short2_t, floor2);
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, f));
}

template <int N>
__device__ __forceinline__ void wait_loads() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// WM x WN computing waves of MT x NT 16 x 16 tiles, plus the loading waves.
// A unit is kSteps MFMA steps of 32 channels; D buffers form a ring, so D - 1
// units are in flight (the layers this kernel serves multiply little per byte:
// what bounds them is memory latency times the bytes LDS can hold in flight).
// LDS per buffer: weights [kSteps * 4 chunks][NF][16 bytes], then pixels
// [kSteps][2 planes of 16 channels][BM][32 bytes].
template <bool BF, int WM, int WN, int MT, int NT, int kSteps, int D>
__global__ __launch_bounds__((WM * WN + kLoaderWaves) * 64) void conv1x1_pipe_kernel(
    const PipeParams p) {
  static_assert(NT % 2 == 0, "filter tiles are stored in pairs");
  constexpr int NWC = WM * WN;
  constexpr int NL = kLoaderWaves * 64;
  constexpr int NF = WN * NT * 16;
  constexpr int BM = WM * MT * 16;
  constexpr int kWeightSlots = kSteps * 4 * NF;
  constexpr int kWeightLoads = (kWeightSlots + NL - 1) / NL;
  constexpr int kWeightBytes = kWeightLoads * NL * 16;
  constexpr int kPixelSlots = kSteps * 2 * BM * 2;
  constexpr int kPixelLoads = kPixelSlots / NL;
  static_assert(kPixelSlots % NL == 0, "whole waves of pixel loads");
  constexpr int kBufBytes = kWeightBytes + kPixelSlots * 16;
  constexpr int kWStep = 4 * NF * 16;          // bytes of weights per 32-channel step
  constexpr int kPStep = 2 * BM * 32;          // bytes of pixels per 32-channel step
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LdsPtr)lds;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  const int wg = blockIdx.x;
  const int t_begin = wg * p.tiles_q + min(wg, p.tiles_r);
  const int t_end = t_begin + p.tiles_q + (wg < p.tiles_r ? 1 : 0);
  const int n_units = (t_end - t_begin) * p.n_units;
  if (n_units <= 0) return;

  if (wave >= NWC) {
    // ================================ loading waves ================================
    const int lw = wave - NWC;
    const i32x4 xrsrc = pipe_rsrc(p.x, p.x_bytes), wrsrc = pipe_rsrc(p.w, p.w_bytes);
    const i32x4 x2rsrc = pipe_rsrc(p.x2, p.x2_bytes);
    // pixel slot s = ((step * 2 + plane) * BM + pixel) * 2 + half
    uint32_t poff[kPixelLoads];    // byte offset in x of the slot's pixel; kOutside: none
    uint32_t poff2[kPixelLoads];   // likewise in x2
    int l_f0 = 0;
    auto setup_load = [&](int tile) {
      const int strip = div_by(tile, p.divF);
      l_f0 = (tile - strip * p.fgroups) * NF;
      const int m0 = strip * BM;
#pragma unroll
      for (int i = 0; i < kPixelLoads; ++i) {
        const int s = (i * kLoaderWaves + lw) * 64 + lane;
        const int m = m0 + ((s >> 1) % BM);
        uint32_t off = kOutside, off2 = kOutside;
        if (m < p.M) {
          if (p.plain) off = (uint32_t)m * (uint32_t)(p.xcs * 2);
          if (!p.plain || p.x2) {
            const int n = div_by(m, p.divPQ), rem = m - n * p.PQ;
            const int pp = div_by(rem, p.divQ), qq = rem - pp * p.Q;
            if (!p.plain)
              off = (uint32_t)(((n * p.H + pp * p.stride) * p.W + qq * p.stride) * p.xcs) * 2u;
            off2 = (uint32_t)(((n * p.H2 + pp * p.stride2) * p.W2 + qq * p.stride2) * p.xcs2) * 2u;
          }
        }
        poff[i] = off;
        poff2[i] = off2;
      }
    };
    auto issue = [&](int unit, uint32_t dst) {
#pragma unroll
      for (int i = 0; i < kWeightLoads; ++i) {
        const int sbase = (i * kLoaderWaves + lw) * 64, s = sbase + lane;
        const int row = s / NF, f = s - row * NF;          // row = step * 4 + chunk of the step
        const int cc = unit * (kSteps * 4) + row;
        const bool ok = s < kWeightSlots && cc < p.cpt && l_f0 + f < p.Kp;
        const uint32_t off = ok ? (uint32_t)(cc * p.Kp + l_f0 + f) * 16u : kOutside;
        pipe_load_to_lds(wrsrc, off, dst + sbase * 16);
      }
#pragma unroll
      for (int i = 0; i < kPixelLoads; ++i) {
        const int sbase = (i * kLoaderWaves + lw) * 64, s = sbase + lane;
        const int half = s & 1, sp = (s >> 1) / BM;        // sp = step * 2 + plane
        const int chunk = unit * (kSteps * 4) + sp * 2 + half;
        // the 64 slots of one load lie in one plane of 16 channels, and the second
        // tensor starts at a multiple of 32 channels: one tensor per load
        const int first = __builtin_amdgcn_readfirstlane(unit * (kSteps * 4) + (sbase >> 1) / BM * 2);
        if (first < p.split) {
          const uint32_t off = chunk * 8 < p.xcs ? poff[i] + (uint32_t)chunk * 16u : kOutside;
          pipe_load_to_lds(xrsrc, off, dst + kWeightBytes + sbase * 16);
        } else {
          const int c2 = chunk - p.split;
          const uint32_t off = c2 * 8 < p.xcs2 ? poff2[i] + (uint32_t)c2 * 16u : kOutside;
          pipe_load_to_lds(x2rsrc, off, dst + kWeightBytes + sbase * 16);
        }
      }
    };

    constexpr int L = kWeightLoads + kPixelLoads;   // loads per thread and unit
    static_assert((D - 2) * L <= 63, "the load counter holds 63");
    int l_tile = t_begin, l_unit = 0;
    int issued = 0;
    auto issue_next = [&]() {   // unit number `issued` of this workgroup into its ring slot
      if (l_unit == 0) setup_load(l_tile);
      issue(l_unit, lds_base + (uint32_t)(issued % D) * (uint32_t)kBufBytes);
      if (++l_unit == p.n_units) { l_unit = 0; ++l_tile; }
      ++issued;
    };
    // before barrier u: unit u has landed, up to D - 2 younger units may be in flight
    auto wait_for = [&](int u) {
      const int younger = issued - 1 - u;
      if (D >= 4 && younger >= 2) wait_loads<(D >= 4 ? 2 : 0) * L>();
      else if (D >= 3 && younger >= 1) wait_loads<(D >= 3 ? 1 : 0) * L>();
      else wait_loads<0>();
    };
    for (int k = 0; k < D - 1 && issued < n_units; ++k) issue_next();
    wait_for(0);
    for (int u = 0; u < n_units; ++u) {
      __syncthreads();   // unit u is in LDS; the computing waves have finished unit u - 1
      if (issued < n_units) issue_next();   // into the slot unit u - 1 has left
      if (u + 1 < n_units) wait_for(u + 1);
    }
    return;
  }

  // ================================ computing waves ================================
  const int li = lane & 15, g = lane >> 4;
  const int wm = wave % WM, wn = wave / WM;
  const __amdgpu_buffer_rsrc_t yrsrc =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.res), 0, p.res_bytes, 0x00020000);
  constexpr int NP = NT / 2;
  uint32_t yoff[MT], roff[MT];
  int c_f0 = 0;
  f32x4 acc[MT][NT], bias4[NT];
  u32x4 rvw[MT][NP];   // shortcut values, fetched during the last unit of a tile
  int rin[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
    rin[mt] = ((wm * MT + mt) * 16 + li) * 32 + (g >> 1) * (BM * 32) + (g & 1) * 16;
  auto setup_compute = [&](int tile) {
    const int strip = div_by(tile, p.divF);
    c_f0 = (tile - strip * p.fgroups) * NF;
    const int m0 = strip * BM;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = m0 + (wm * MT + mt) * 16 + li;
      yoff[mt] = kOutside;
      roff[mt] = kOutside;
      if (m < p.M) {
        yoff[mt] = (uint32_t)m * (uint32_t)(p.ycs * 2);
        if (p.plain) {
          roff[mt] = (uint32_t)m * (uint32_t)(p.rcs * 2);
        } else if (p.res) {
          const int n = div_by(m, p.divPQ), rem = m - n * p.PQ;
          const int pp = div_by(rem, p.divQ), qq = rem - pp * p.Q;
          roff[mt] = (uint32_t)(((n * p.rH + pp * p.rss) * p.rW + qq * p.rss) * p.rcs) * 2u;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int k0 = min(c_f0 + (wn * NT + t) * 16, p.Kp - 16) + g * 4;
      bias4[t] = *reinterpret_cast<const f32x4*>(p.bias + k0);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  };
  const int a_lane = g * (NF * 16) + (wn * NT * 16 + li) * 16;
  const int k_pair = wn * NT * 16 + (g & 1) * 16 + (g >> 1) * 8;
  const uint32_t floor2 = p.relu ? 0u : 0x80008000u;

  int c_tile = t_begin, c_unit = 0;
  for (int u = 0; u < n_units; ++u) {
    __syncthreads();   // unit u is in LDS
    if (c_unit == 0) setup_compute(c_tile);
    const bool last = c_unit == p.n_units - 1;
    if (last && p.res) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int pr = 0; pr < NP; ++pr) {
          const int rc = c_f0 + k_pair + pr * 32 - p.roff;
          const uint32_t off = (rc >= 0 && rc < p.rcs) ? roff[mt] + (uint32_t)rc * 2u : kOutside;
          rvw[mt][pr] = __builtin_amdgcn_raw_buffer_load_b128(rrsrc, off, 0, 0);
        }
    }
    const char* wts = lds + (u % D) * kBufBytes;
    const char* pix = wts + kWeightBytes;
    uint4 a[2][NT], b[2][MT];
    auto operands = [&](int step, uint4* av, uint4* bv) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
        av[t] = *reinterpret_cast<const uint4*>(wts + a_lane + step * kWStep + t * 256);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        bv[mt] = *reinterpret_cast<const uint4*>(pix + rin[mt] + step * kPStep);
    };
    operands(0, a[0], b[0]);
#pragma unroll
    for (int step = 0; step < kSteps; ++step) {
      if (step + 1 < kSteps) operands(step + 1, a[(step + 1) & 1], b[(step + 1) & 1]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[mt][t] = mfma_16x16x32<BF>(a[step & 1][t], b[step & 1][mt], acc[mt][t]);
    }
    if (last) {
      auto finish = [&](const f32x4& av, const f32x4& bv, uint32_t r0, uint32_t r1) {
        float v[4] = {av[0] + bv[0], av[1] + bv[1], av[2] + bv[2], av[3] + bv[3]};
        if (p.res) {
          v[0] += to_float<BF>((uint16_t)(r0 & 0xffffu));
          v[1] += to_float<BF>((uint16_t)(r0 >> 16));
          v[2] += to_float<BF>((uint16_t)(r1 & 0xffffu));
          v[3] += to_float<BF>((uint16_t)(r1 >> 16));
        }
        u32x2 o;
        o[0] = pipe_clamp(pack2<BF>(v[0], v[1]), floor2);
        o[1] = pipe_clamp(pack2<BF>(v[2], v[3]), floor2);
        return o;
      };
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int pr = 0; pr < NP; ++pr) {
          const int t = 2 * pr;
          uint32_t ra0 = 0, ra1 = 0, rb0 = 0, rb1 = 0;
          if (p.res) {
            const u32x4 x4 = rvw[mt][pr];
            const auto s0 = __builtin_amdgcn_permlane16_swap(x4[0], x4[2], false, false);
            const auto s1 = __builtin_amdgcn_permlane16_swap(x4[1], x4[3], false, false);
            ra0 = s0[0]; ra1 = s1[0];
            rb0 = s0[1]; rb1 = s1[1];
          }
          const u32x2 oa = finish(acc[mt][t], bias4[t], ra0, ra1);
          const u32x2 ob = finish(acc[mt][t + 1], bias4[t + 1], rb0, rb1);
          const auto w0 = __builtin_amdgcn_permlane16_swap(oa[0], ob[0], false, false);
          const auto w1 = __builtin_amdgcn_permlane16_swap(oa[1], ob[1], false, false);
          const u32x4 o4 = {w0[0], w1[0], w0[1], w1[1]};
          const int k0 = c_f0 + k_pair + pr * 32;
          const uint32_t off = k0 < p.ycs ? yoff[mt] + (uint32_t)k0 * 2u : kOutside;
          __builtin_amdgcn_raw_buffer_store_b128(o4, yrsrc, off, 0, 0);
        }
      }
      c_unit = 0;
      ++c_tile;
    } else {
      ++c_unit;
    }
  }
}

struct PipeTile {
  int WM, WN, MT, NT, steps, depth;
  const char* name;
};
constexpr PipeTile kPipeTiles[] = {
    {2, 2, 4, 4, 2, 4, "conv1x1p_128x128"},
    {4, 1, 2, 4, 4, 3, "conv1x1p_128x64"},
    {2, 2, 2, 2, 4, 4, "conv1x1p_64x64"},
};
constexpr int kNumPipeTiles = sizeof(kPipeTiles) / sizeof(kPipeTiles[0]);

int pipe_compute_units() {
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

struct PipePlan {
  int tile;
  int units;
  int fgroups;
  int64_t tiles;
  size_t lds_bytes;
  int grid;
};

// The tile with the least estimated time; the tuning switch pipe_tile=<index> forces one.
bool plan_pipe(const Conv16Params& c, PipePlan* out) {
  if (tuning_off("conv1x1_pipe")) return false;
  if (c.S != 1 || c.nchunk != c.cpt || c.pad != 0 || (c.stride != 1 && c.stride != 2)) return false;
  if (c.roff % 8 != 0) return false;
  if (c.cpt < 16) return false;   // fewer than 128 channels: one unit, nothing to pipeline
  const int forced = tuning_int("pipe_tile", -1);
  const int cus = pipe_compute_units();
  double best = 1e30;
  bool found = false;
  for (int i = 0; i < kNumPipeTiles; ++i) {
    const PipeTile& t = kPipeTiles[i];
    const int BM = t.WM * t.MT * 16, NF = t.WN * t.NT * 16;
    const int NL = kLoaderWaves * 64;
    const int units = (c.cpt + 4 * t.steps - 1) / (4 * t.steps);
    const size_t wbytes = (size_t)((t.steps * 4 * NF + NL - 1) / NL) * NL * 16;
    const size_t buf = wbytes + (size_t)t.steps * 2 * BM * 2 * 16;
    if (t.depth * buf > kPipeLdsLimit) continue;
    const int fgroups = (c.Kp + NF - 1) / NF;
    const int64_t tiles = ((int64_t)c.M + BM - 1) / BM * fgroups;
    if (tiles >= (int64_t(1) << 30)) continue;
    const int grid = (int)std::min<int64_t>(tiles, cus);
    // clocks per unit: loads (bounded by the bytes in flight over the memory
    // latency, about 4000 clocks, and by 40 bytes per clock) against MFMA + LDS reads
    const double load = std::max((double)buf / 40.0, 4000.0 / (t.depth - 1));
    const double mfma = t.steps * t.MT * t.NT * 16.0 + t.steps * (t.MT + t.NT) * 4 * 5.4;
    const double per_tile = units * (std::max(load, mfma) + 150.0) + 400.0 + BM * NF / 16.0;
    const double cost = 6000.0 + (double)((tiles + grid - 1) / grid) * per_tile;
    if (i == forced || cost < best) {
      best = i == forced ? -1.0 : cost;
      out->tile = i;
      out->units = units;
      out->fgroups = fgroups;
      out->tiles = tiles;
      out->lds_bytes = t.depth * buf;
      out->grid = grid;
      found = true;
    }
  }
  return found;
}

template <bool BF, int WM, int WN, int MT, int NT, int KS, int D>
fupr_status launch_pipe(const PipeParams& p, const PipePlan& plan, hipStream_t st) {
  static std::once_flag once;
  static hipError_t status = hipSuccess;
  std::call_once(once, [] {
    status =
        hipFuncSetAttribute(reinterpret_cast<const void*>(&conv1x1_pipe_kernel<BF, WM, WN, MT, NT, KS, D>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPipeLdsLimit);
  });
  if (status != hipSuccess) return FUPR_ERR_LAUNCH;
  hipLaunchKernelGGL((conv1x1_pipe_kernel<BF, WM, WN, MT, NT, KS, D>), dim3((unsigned)plan.grid),
                     dim3((WM * WN + kLoaderWaves) * 64), plan.lds_bytes, st, p);
  return launch_status("conv1x1_pipe_kernel");
}

template <bool BF>
fupr_status dispatch_pipe(const PipeParams& p, const PipePlan& plan, hipStream_t st) {
  switch (plan.tile) {
    case 0: return launch_pipe<BF, 2, 2, 4, 4, 2, 4>(p, plan, st);
    case 1: return launch_pipe<BF, 4, 1, 2, 4, 4, 3>(p, plan, st);
    default: return launch_pipe<BF, 2, 2, 2, 2, 4, 4>(p, plan, st);
  }
}

}  // namespace

bool conv1x1_pipe_applies(const Conv16Params& c) {
  PipePlan plan;
  return plan_pipe(c, &plan);
}

const char* conv1x1_pipe_name(const Conv16Params& c) {
  PipePlan plan;
  return plan_pipe(c, &plan) ? kPipeTiles[plan.tile].name : "conv1x1p";
}

fupr_status launch_conv1x1_pipe(const Conv16Params& c, int N, bool bf16, void* stream) {
  PipePlan plan;
  if (!plan_pipe(c, &plan)) return FUPR_ERR_LIMIT;
  PipeParams p{};
  p.x = c.x; p.w = c.w; p.bias = c.bias; p.res = c.res; p.y = c.y;
  const uint64_t y_bytes = (uint64_t)c.M * c.ycs * 2;
  const uint64_t res_bytes = c.res ? (uint64_t)N * c.rH * c.rW * c.rcs * 2 : 0;
  if ((uint64_t)c.x_bytes >= kOutside || y_bytes >= kOutside || res_bytes >= kOutside ||
      (uint64_t)c.x2_bytes >= kOutside)
    return FUPR_ERR_LIMIT;
  p.x_bytes = c.x_bytes; p.w_bytes = c.w_bytes;
  p.y_bytes = (uint32_t)y_bytes; p.res_bytes = (uint32_t)res_bytes;
  p.H = c.H; p.W = c.W; p.xcs = c.xcs;
  p.P = c.P; p.Q = c.Q; p.PQ = c.PQ; p.M = c.M; p.ycs = c.ycs;
  p.stride = c.stride;
  p.Kp = c.Kp; p.cpt = c.cpt;
  p.n_units = plan.units;
  p.rH = c.rH; p.rW = c.rW; p.rcs = c.rcs; p.rss = c.rss; p.roff = c.roff;
  p.relu = c.relu;
  p.plain = c.stride == 1 && (!c.res || (c.rss == 1 && c.rH == c.P && c.rW == c.Q));
  p.fgroups = plan.fgroups;
  p.tiles = (int)plan.tiles;
  p.tiles_q = p.tiles / plan.grid;
  p.tiles_r = p.tiles % plan.grid;
  p.divPQ = fast_div(c.PQ);
  p.divQ = fast_div(c.Q);
  p.divF = fast_div(plan.fgroups);
  p.x2 = c.x2; p.x2_bytes = c.x2_bytes;
  p.split = c.x2 ? c.split : (1 << 30);
  p.H2 = c.H2; p.W2 = c.W2; p.xcs2 = c.xcs2; p.stride2 = c.stride2;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  return bf16 ? dispatch_pipe<true>(p, plan, st) : dispatch_pipe<false>(p, plan, st);
}

}  // namespace fupr
