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
// persistent, so the loads of the next tile fly during the last units of the
// current one.  Tiles are numbered strip of pixels first, group of filters
// second, and the workgroups of one XCD take consecutive tiles at the same
// time: the filter groups of a strip read its pixels from that XCD's L2 while
// they are there, not once per group from memory.
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
  int xcd_order;         // 1: workgroups of one XCD take consecutive tiles; 0: a range of tiles each
  int tiles_q, tiles_r;  // tiles / grid, tiles % grid
  FastDiv divPQ, divQ, divF;
  // second input tensor: chunks from `split` on come from x2 at spatial stride
  // stride2 (split is a multiple of 8; 1 << 30 when there is no second tensor)
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

// What the two kernels below share.  A tile is BM output pixels x NF filters; a
// unit is kSteps steps of 32 channels of it; D buffers form a ring, so D - 1
// units are in flight (the layers this kernel serves multiply little per byte:
// what bounds them is memory latency times the bytes LDS can hold in flight).
// LDS per buffer: weights [kSteps * 4 chunks][NF][16 bytes], then pixels
// [kSteps / 2][BM][128 bytes]: 64 channels of a pixel side by side, so that one
// load instruction fetches whole 128-byte lines of 8 pixels; the eight 16-byte
// pieces of a row are stored at piece ^ ((pixel >> 1) & 7), which keeps the
// operand reads of 16 or 32 lanes (pixels 128 bytes apart) off each other's banks.
template <int BM_, int NF_, int kSteps_, int D_>
struct PipeGeom {
  static constexpr int BM = BM_, NF = NF_, kSteps = kSteps_, D = D_;
  static constexpr int NL = kLoaderWaves * 64;
  static constexpr int kWeightSlots = kSteps * 4 * NF;
  static constexpr int kWeightLoads = (kWeightSlots + NL - 1) / NL;
  static constexpr int kWeightBytes = kWeightLoads * NL * 16;
  static constexpr int kPixelSlots = kSteps * 2 * BM * 2;
  static constexpr int kPixelLoads = kPixelSlots / NL;
  static_assert(kPixelSlots % NL == 0, "whole waves of pixel loads");
  static constexpr int kBufBytes = kWeightBytes + kPixelSlots * 16;
  static_assert(kSteps % 2 == 0, "pixels are stored 64 channels at a time");
  static constexpr int kWStep = 4 * NF * 16;   // bytes of weights per 32-channel step
  static constexpr int kPHalf = BM * 128;      // bytes of pixels per 64 channels
};

// The tiles of a workgroup: t_begin, t_begin + t_step, ... (t_count of them).
// Workgroups go to the XCDs in turn, so with a grid of 8 n workgroups those
// numbered x, x + 8, ... share XCD x and take n consecutive tiles per round.
struct PipeTiles {
  int t_begin, t_step, t_count;
};
__device__ __forceinline__ PipeTiles pipe_tiles_of_workgroup(const PipeParams& p) {
  const int wg = blockIdx.x, grid = gridDim.x;
  PipeTiles t;
  if (p.xcd_order) {
    t.t_begin = (grid & 7) == 0 ? (wg & 7) * (grid >> 3) + (wg >> 3) : wg;
    t.t_step = grid;
    t.t_count = p.tiles_q + (t.t_begin < p.tiles_r ? 1 : 0);
  } else {
    t.t_begin = wg * p.tiles_q + min(wg, p.tiles_r);
    t.t_step = 1;
    t.t_count = p.tiles_q + (wg < p.tiles_r ? 1 : 0);
  }
  return t;
}

// A loading wave (number lw of kLoaderWaves): all units of the workgroup's tiles,
// global -> LDS, one barrier per unit with the computing waves.
template <typename G>
__device__ __forceinline__ void pipe_loader(const PipeParams& p, uint32_t lds_base, int lw, int lane,
                                            int t_begin, int t_step, int n_units) {
  constexpr int BM = G::BM, NF = G::NF, kSteps = G::kSteps, D = G::D;
  constexpr int kWeightSlots = G::kWeightSlots, kWeightLoads = G::kWeightLoads;
  constexpr int kWeightBytes = G::kWeightBytes, kPixelLoads = G::kPixelLoads, kBufBytes = G::kBufBytes;
  const i32x4 xrsrc = pipe_rsrc(p.x, p.x_bytes), wrsrc = pipe_rsrc(p.w, p.w_bytes);
  const i32x4 x2rsrc = pipe_rsrc(p.x2, p.x2_bytes);
  // pixel slot s = ((64-channel block * BM) + pixel) * 8 + stored piece
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
      const int m = m0 + ((s >> 3) % BM);
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
      const int pixel = (s >> 3) % BM;
      const int piece = (s & 7) ^ ((pixel >> 1) & 7);
      // the 64 slots of one load are 64 channels of 8 pixels, and the second tensor
      // starts at a multiple of 64 channels: one tensor per load
      const int first = __builtin_amdgcn_readfirstlane(unit * (kSteps * 4) + (sbase >> 3) / BM * 8);
      const int chunk = first + piece;
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
    if (++l_unit == p.n_units) { l_unit = 0; l_tile += t_step; }
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
}

// WM x WN computing waves of MT x NT tiles of 16 x 16 (MFMA 16 x 16 x 32), plus the
// loading waves.
template <bool BF, int WM, int WN, int MT, int NT, int kSteps, int D>
__global__ __launch_bounds__((WM * WN + kLoaderWaves) * 64) void conv1x1_pipe_kernel(
    const PipeParams p) {
  static_assert(NT % 2 == 0, "filter tiles are stored in pairs");
  using G = PipeGeom<WM * MT * 16, WN * NT * 16, kSteps, D>;
  constexpr int NWC = WM * WN;
  constexpr int NF = G::NF, BM = G::BM;
  constexpr int kWeightBytes = G::kWeightBytes, kBufBytes = G::kBufBytes;
  constexpr int kWStep = G::kWStep, kPHalf = G::kPHalf;
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LdsPtr)lds;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const PipeTiles tl = pipe_tiles_of_workgroup(p);
  const int t_begin = tl.t_begin, t_step = tl.t_step;
  const int n_units = tl.t_count * p.n_units;
  if (n_units <= 0) return;

  if (wave >= NWC) {
    pipe_loader<G>(p, lds_base, wave - NWC, lane, t_begin, t_step, n_units);
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
    rin[mt] = ((wm * MT + mt) * 16 + li) * 128 + ((g ^ ((li >> 1) & 7)) * 16);   // even steps; odd: ^ 64
  // the tile's pixel offsets; its accumulators start at zero
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
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  };
  const int a_lane = g * (NF * 16) + (wn * NT * 16 + li) * 16;
  const int k_pair = wn * NT * 16 + (g & 1) * 16 + (g >> 1) * 8;
  const uint32_t floor2 = p.relu ? 0u : 0x80008000u;

  // The steps of all units form one stream: the operands of a step are read from
  // LDS while the step before it multiplies, also across units.  The barrier that
  // says unit u + 1 has landed therefore stands before the last step of unit u
  // multiplies (that step's operands are in registers by then, so the loading
  // waves may overwrite unit u from this barrier on, as before).
  uint4 a[2][NT], b[2][MT];
  auto operands = [&](const char* wts, int step, uint4* av, uint4* bv) {
    const char* pix = wts + kWeightBytes;
#pragma unroll
    for (int t = 0; t < NT; ++t)
      av[t] = *reinterpret_cast<const uint4*>(wts + a_lane + step * kWStep + t * 256);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      bv[mt] = *reinterpret_cast<const uint4*>(pix + (rin[mt] ^ ((step & 1) * 64)) + (step >> 1) * kPHalf);
  };
  int c_tile = t_begin, c_unit = 0;
  __syncthreads();   // unit 0 is in LDS
  setup_compute(c_tile);
  operands(lds, 0, a[0], b[0]);
  for (int u = 0; u < n_units; ++u) {
    const bool last = c_unit == p.n_units - 1;
    if (last) {   // what the epilogue adds, fetched while the last unit multiplies
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int k0 = min(c_f0 + (wn * NT + t) * 16, p.Kp - 16) + g * 4;
        bias4[t] = *reinterpret_cast<const f32x4*>(p.bias + k0);
      }
      if (p.res) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int pr = 0; pr < NP; ++pr) {
            const int rc = c_f0 + k_pair + pr * 32 - p.roff;
            const uint32_t off = (rc >= 0 && rc < p.rcs) ? roff[mt] + (uint32_t)rc * 2u : kOutside;
            rvw[mt][pr] = __builtin_amdgcn_raw_buffer_load_b128(rrsrc, off, 0, 0);
          }
      }
    }
    const char* wts = lds + (u % D) * kBufBytes;
#pragma unroll
    for (int step = 0; step < kSteps; ++step) {
      if (step + 1 < kSteps) {
        operands(wts, step + 1, a[(step + 1) & 1], b[(step + 1) & 1]);
      } else if (u + 1 < n_units) {
        __syncthreads();   // unit u + 1 is in LDS
        operands(lds + ((u + 1) % D) * kBufBytes, 0, a[0], b[0]);
      }
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
      c_tile += t_step;
      if (u + 1 < n_units) setup_compute(c_tile);
    } else {
      ++c_unit;
    }
  }
}

// The same pipeline on the 32 x 32 x 16 MFMA (half as many MFMA instructions and
// accumulator reads per flop), with eight computing waves in the tiles that are
// selected: WM x WN computing waves, each
// owning MT pixel tiles x NT filter tiles of 32 x 32 (16 accumulator registers each).
// LDS layout and loading waves are shared with conv1x1_pipe_kernel.  A step is 16
// channels here: lane (index j = lane % 32, half h = lane / 32) reads chunk 2 * step + h
// of filter j and piece 2 * step + h of pixel j.  The operands of a step are read PD
// steps ahead of its MFMAs (2 or 4 register sets in turn), also across units: the barrier
// that says unit u + 1 has landed stands PD steps before the end of unit u, and every
// read of unit u has been issued before it.  The layer's biases are staged in LDS once
// (behind the ring of buffers) and a tile's accumulators start from them, so the
// epilogue holds no bias registers.  A finished tile holds, per lane, channels
// 8 b + 4 h .. + 3 (b = 0 .. 3) of pixel j; the two lanes of a pixel exchange halves
// (v_permlane32_swap) so that each stores 16 bytes: channels 16 pr + 8 h .. + 7.
constexpr int kPipeBiasBytes = 8192;   // up to 2048 filters per layer in the 32 x 32 kernel
template <bool BF, int WM, int WN, int MT, int NT, int kSteps, int D, int PD>
__global__ __launch_bounds__((WM * WN + kLoaderWaves) * 64) void conv1x1_pipe32_kernel(
    const PipeParams p) {
  using G = PipeGeom<WM * MT * 32, WN * NT * 32, kSteps, D>;
  constexpr int NWC = WM * WN;
  constexpr int NF = G::NF;
  constexpr int kWeightBytes = G::kWeightBytes, kBufBytes = G::kBufBytes, kPHalf = G::kPHalf;
  constexpr int S = 2 * kSteps;                // steps of 16 channels per unit
  constexpr int SETS = PD == 1 ? 2 : 4;        // operand register sets
  static_assert((PD == 1 || PD == 2) && S % SETS == 0, "operand register sets in turn");
  constexpr int kWHalf = 2 * NF * 16;          // bytes of weights per 16-channel step
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LdsPtr)lds;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const PipeTiles tl = pipe_tiles_of_workgroup(p);
  const int t_begin = tl.t_begin, t_step = tl.t_step;
  const int n_units = tl.t_count * p.n_units;
  if (n_units <= 0) return;

  if (wave >= NWC) {
    pipe_loader<G>(p, lds_base, wave - NWC, lane, t_begin, t_step, n_units);
    return;
  }

  // ================================ computing waves ================================
  const int j = lane & 31, h = lane >> 5;
  const int wm = wave % WM, wn = wave / WM;
  const __amdgpu_buffer_rsrc_t yrsrc =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.res), 0, p.res_bytes, 0x00020000);
  uint32_t yoff[MT], roff[MT];
  int c_f0 = 0;
  f32x16 acc[MT][NT];
  u32x4 rvw[MT][NT][2];   // shortcut values, fetched during the last unit of a tile
  const float* lds_bias = reinterpret_cast<const float*>(lds + D * kBufBytes);
  int rin[MT];            // step 0 of a 64-channel block; step s of it: ^ (s * 32)
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
    rin[mt] = ((wm * MT + mt) * 32 + j) * 128 + ((h ^ ((j >> 1) & 7)) * 16);
  auto setup_compute = [&](int tile) {
    const int strip = div_by(tile, p.divF);
    c_f0 = (tile - strip * p.fgroups) * NF;
    const int m0 = strip * G::BM;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = m0 + (wm * MT + mt) * 32 + j;
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
    // the accumulators start from the biases of their filters
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int kt = c_f0 + (wn * NT + t) * 32;   // first filter of this 32-row tile
#pragma unroll
      for (int bb = 0; bb < 4; ++bb) {
        const f32x4 b4 = *reinterpret_cast<const f32x4*>(lds_bias + min(kt + 8 * bb + 4 * h, p.Kp - 4));
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[mt][t][4 * bb + i] = b4[i];
      }
    }
  };
  const int a_lane = h * (NF * 16) + (wn * NT * 32 + j) * 16;
  const int k_lane = wn * NT * 32 + h * 8;   // first channel of this lane's 16 bytes, pair 0 of tile 0
  const uint32_t floor2 = p.relu ? 0u : 0x80008000u;

  uint4 a[SETS][NT], b[SETS][MT];
  auto operands = [&](const char* wts, int step, uint4* av, uint4* bv) {
    const char* pix = wts + kWeightBytes + (step >> 2) * kPHalf;
#pragma unroll
    for (int t = 0; t < NT; ++t)
      av[t] = *reinterpret_cast<const uint4*>(wts + a_lane + step * kWHalf + t * 512);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      bv[mt] = *reinterpret_cast<const uint4*>(pix + (rin[mt] ^ ((step & 3) * 32)));
  };
  int c_tile = t_begin, c_unit = 0;
  // the computing waves stage the biases while the first unit is on its way
  for (int i = wave * 64 + lane; i < p.Kp; i += NWC * 64)
    reinterpret_cast<float*>(lds + D * kBufBytes)[i] = p.bias[i];
  __syncthreads();   // unit 0 and the biases are in LDS
  setup_compute(c_tile);
#pragma unroll
  for (int s0 = 0; s0 < PD; ++s0) operands(lds, s0, a[s0], b[s0]);
  for (int u = 0; u < n_units; ++u) {
    const bool last = c_unit == p.n_units - 1;
    if (last) {   // what the epilogue adds, fetched while the last unit multiplies
      if (p.res) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
              const int rc = c_f0 + k_lane + t * 32 + pr * 16 - p.roff;
              const uint32_t off = (rc >= 0 && rc < p.rcs) ? roff[mt] + (uint32_t)rc * 2u : kOutside;
              rvw[mt][t][pr] = __builtin_amdgcn_raw_buffer_load_b128(rrsrc, off, 0, 0);
            }
      }
    }
    const char* wts = lds + (u % D) * kBufBytes;
    const char* next = lds + ((u + 1) % D) * kBufBytes;
#pragma unroll
    for (int step = 0; step < S; ++step) {
      const int ns = step + PD;   // the step whose operands are read now
      if (ns < S) {
        operands(wts, ns, a[ns % SETS], b[ns % SETS]);
      } else if (u + 1 < n_units) {
        if (ns == S) __syncthreads();   // unit u + 1 is in LDS
        operands(next, ns - S, a[ns % SETS], b[ns % SETS]);
      }
      // the reads stay in front of this step's MFMAs: left alone, the scheduler sinks
      // every read to just before its use and each MFMA waits out an LDS round trip
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[mt][t] = mfma_32x32x16<BF>(a[step % SETS][t], b[step % SETS][mt], acc[mt][t]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (!last) {
      ++c_unit;
      continue;
    }
    // ---- epilogue: bias, shortcut, ReLU, one rounding, 16-byte stores ----
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
          // shortcut values into the accumulators' layout: the lanes of a pixel exchange halves
          uint32_t ra[2] = {0u, 0u}, rb[2] = {0u, 0u};
          if (p.res) {
            const u32x4 r4 = rvw[mt][t][pr];
            const auto s0 = __builtin_amdgcn_permlane32_swap(r4[0], r4[2], false, false);
            const auto s1 = __builtin_amdgcn_permlane32_swap(r4[1], r4[3], false, false);
            ra[0] = s0[0]; ra[1] = s1[0];   // group 2 pr
            rb[0] = s0[1]; rb[1] = s1[1];   // group 2 pr + 1
          }
          auto finish = [&](int bb, const uint32_t* r) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = acc[mt][t][4 * bb + i];
            if (p.res) {
              v[0] += to_float<BF>((uint16_t)(r[0] & 0xffffu));
              v[1] += to_float<BF>((uint16_t)(r[0] >> 16));
              v[2] += to_float<BF>((uint16_t)(r[1] & 0xffffu));
              v[3] += to_float<BF>((uint16_t)(r[1] >> 16));
            }
            u32x2 o;
            o[0] = pipe_clamp(pack2<BF>(v[0], v[1]), floor2);
            o[1] = pipe_clamp(pack2<BF>(v[2], v[3]), floor2);
            return o;
          };
          const u32x2 oa = finish(2 * pr, ra), ob = finish(2 * pr + 1, rb);
          const auto w0 = __builtin_amdgcn_permlane32_swap(oa[0], ob[0], false, false);
          const auto w1 = __builtin_amdgcn_permlane32_swap(oa[1], ob[1], false, false);
          const u32x4 o4 = {w0[0], w1[0], w0[1], w1[1]};
          const int k0 = c_f0 + k_lane + t * 32 + pr * 16;
          const uint32_t off = k0 < p.ycs ? yoff[mt] + (uint32_t)k0 * 2u : kOutside;
          __builtin_amdgcn_raw_buffer_store_b128(o4, yrsrc, off, 0, 0);
        }
    c_unit = 0;
    c_tile += t_step;
    if (u + 1 < n_units) setup_compute(c_tile);
  }
}

struct PipeTile {
  int WM, WN, MT, NT, steps, depth;
  const char* name;
  bool wide;   // MFMA tiles of 32 x 32 (conv1x1_pipe32_kernel), else 16 x 16
};
constexpr PipeTile kPipeTiles[] = {
    {2, 2, 4, 4, 2, 4, "conv1x1p_128x128", false},
    {4, 1, 2, 4, 4, 3, "conv1x1p_128x64", false},
    {2, 2, 2, 2, 4, 4, "conv1x1p_64x64", false},
    {2, 2, 2, 2, 2, 4, "conv1x1q_128x128", true},
    {2, 4, 2, 2, 2, 3, "conv1x1q_128x256", true},   // before 256 x 128: it wins a tie
    {4, 2, 2, 2, 2, 3, "conv1x1q_256x128", true},
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
  if (c.x2 && c.split % 8 != 0) return false;   // a load fetches 64 channels of one tensor
  if (c.cpt < 16) return false;   // fewer than 128 channels: one unit, nothing to pipeline
  const int forced = tuning_int("pipe_tile", -1);
  const int cus = pipe_compute_units();
  double best = 1e30;
  bool found = false;
  for (int i = 0; i < kNumPipeTiles; ++i) {
    const PipeTile& t = kPipeTiles[i];
    const int edge = t.wide ? 32 : 16;
    const int BM = t.WM * t.MT * edge, NF = t.WN * t.NT * edge;
    const int NL = kLoaderWaves * 64;
    // (four waves of 64 x 64 on the 32 x 32 MFMA: measured equal to tile 0 on every layer)
    if (t.wide && t.WM * t.WN == 4 && i != forced) continue;
    const int units = (c.cpt + 4 * t.steps - 1) / (4 * t.steps);
    const size_t wbytes = (size_t)((t.steps * 4 * NF + NL - 1) / NL) * NL * 16;
    const size_t buf = wbytes + (size_t)t.steps * 2 * BM * 2 * 16;
    const size_t lds_need = t.depth * buf + (t.wide ? kPipeBiasBytes : 0);
    if (lds_need > kPipeLdsLimit) continue;
    if (t.wide && c.Kp * 4 > kPipeBiasBytes) continue;
    // (tiles of two units: 22.1 against 20.9 us for 128 -> 1024 channels at 14 x 14 x 64)
    if (t.wide && units < 4 && i != forced) continue;
    const int fgroups = (c.Kp + NF - 1) / NF;
    const int64_t tiles = ((int64_t)c.M + BM - 1) / BM * fgroups;
    if (tiles >= (int64_t(1) << 30)) continue;
    const int grid = (int)std::min<int64_t>(tiles, cus);
    // clocks per unit: loads (bounded by the bytes in flight over the memory
    // latency, about 4000 clocks, and by 40 bytes per clock) against the MFMAs of
    // the waves that share a SIMD (measured in this kernel: 28 clocks per
    // 16 x 16 x 32, 40 per 32 x 32 x 16); per tile an epilogue of BM x NF / 8 clocks.
    // A strip's pixels are read once per group of filters: a small preference for
    // fewer groups (measured: 116 against 134 us for 320 -> 512 channels at 56 x 56 x 256).
    const double load = std::max((double)buf / 40.0, 4000.0 / (t.depth - 1));
    const double per_wave = t.wide ? 2.0 * t.steps * t.MT * t.NT * 40.0 : t.steps * t.MT * t.NT * 28.0;
    const double mfma = per_wave * (t.WM * t.WN / 4.0);
    const double per_tile = units * (std::max(load, mfma) + 150.0) + 600.0 + BM * NF / 8.0;
    const double cost = (6000.0 + (double)((tiles + grid - 1) / grid) * per_tile) *
                        (1.0 + 0.02 * std::min(fgroups - 1, 3));
    if (i == forced || cost < best) {
      best = i == forced ? -1.0 : cost;
      out->tile = i;
      out->units = units;
      out->fgroups = fgroups;
      out->tiles = tiles;
      out->lds_bytes = lds_need;
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

template <bool BF, int WM, int WN, int MT, int NT, int KS, int D, int PD>
fupr_status launch_pipe32(const PipeParams& p, const PipePlan& plan, hipStream_t st) {
  static std::once_flag once;
  static hipError_t status = hipSuccess;
  std::call_once(once, [] {
    status =
        hipFuncSetAttribute(reinterpret_cast<const void*>(&conv1x1_pipe32_kernel<BF, WM, WN, MT, NT, KS, D, PD>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPipeLdsLimit);
  });
  if (status != hipSuccess) return FUPR_ERR_LAUNCH;
  hipLaunchKernelGGL((conv1x1_pipe32_kernel<BF, WM, WN, MT, NT, KS, D, PD>), dim3((unsigned)plan.grid),
                     dim3((WM * WN + kLoaderWaves) * 64), plan.lds_bytes, st, p);
  return launch_status("conv1x1_pipe32_kernel");
}

template <bool BF>
fupr_status dispatch_pipe(const PipeParams& p, const PipePlan& plan, hipStream_t st) {
  switch (plan.tile) {
    case 3: return launch_pipe32<BF, 2, 2, 2, 2, 2, 4, 2>(p, plan, st);
    case 4: return launch_pipe32<BF, 2, 4, 2, 2, 2, 3, 1>(p, plan, st);
    case 5: return launch_pipe32<BF, 4, 2, 2, 2, 2, 3, 1>(p, plan, st);
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
  // one group of filters: nothing to share, and a contiguous range of strips per
  // workgroup reads memory in longer runs (37.0 against 39.4 us for 1024 -> 227
  // channels at 14 x 14 x 256)
  p.xcd_order = tuning_int("pipe_order", plan.fgroups > 1 ? 1 : 0) != 0;
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
