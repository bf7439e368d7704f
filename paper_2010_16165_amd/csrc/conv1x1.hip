// 1 x 1 convolution (Sec. III: operator k x c x 1 x 1; the bottleneck blocks'
// first and last convolutions and projection shortcuts) as a streaming kernel
// for layers whose filters fit in LDS: these layers move far more bytes than
// they multiply, so the kernel is built around keeping many loads in flight.
//
//   * A workgroup copies its filter group (all channels) and bias into LDS once
//     and then streams pixels; it is persistent and sized so that two fit a
//     compute unit (eight waves).
//   * Each wave works alone on 16-pixel tiles, with no barrier after the copy:
//     lane (pixel, channel group) loads its 16 bytes per 32-channel step straight
//     from global memory in MFMA layout, the filter fragments come from LDS,
//     the epilogue adds the shortcut, applies ReLU, rounds once and stores
//     8 bytes per lane.
//   * The pixel fragments and shortcut values of the wave's next tile are
//     loaded before the current tile is multiplied, so every wave always has a
//     whole tile of loads outstanding.
//   * All global accesses are range-checked buffer accesses: channels past the
//     tensor's stride and pixels past the end read zeros, stores there vanish.
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
constexpr int kStreamLdsLimit = 72 * 1024;   // two workgroups per compute unit
constexpr int kStreamFusedLdsLimit = 80 * 1024;   // likewise, with a second layer's filters

struct StreamParams {
  const uint16_t* x;
  const uint16_t* w;     // [nchunk_pad][Kp][8]
  const float* bias;
  const uint16_t* res;
  uint16_t* y;
  uint32_t x_bytes, w_bytes, y_bytes, res_bytes;
  int H, W, xcs;
  int P, Q, PQ, M, ycs;
  int stride;
  int Kp, cpt, ksteps;
  int rH, rW, rcs, rss, roff;
  int relu;
  int plain;             // pixel m of the output is pixel m of the input and of the shortcut
  // a second 1 x 1 convolution applied to the output tile while it is in registers
  const uint16_t* w2;    // [nchunk_pad2][Kp2][8]; its channels are this layer's filters
  const float* bias2;
  uint16_t* h;           // its output, M pixels x hcs
  uint32_t w2_bytes, h_bytes;
  int Kp2, cpt2, hcs, relu2;
  int w_lds_bytes;       // LDS bytes of the first convolution's filters
  int n_tiles;           // 16-pixel tiles
  // second input tensor: chunks from `split` on come from x2 at spatial stride
  // stride2 (split is a multiple of 8; 1 << 30 when there is no second tensor)
  const uint16_t* x2;
  uint32_t x2_bytes;
  int split, H2, W2, xcs2, stride2;
};

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef void __attribute__((address_space(3)))* LdsPtr;
typedef short short2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t clamp_below2(uint32_t v, uint32_t floor2) {
  const short2_t a = __builtin_bit_cast(short2_t, v), f = __builtin_bit_cast(short2_t, floor2);
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, f));
}

// NT filter tiles of 16 per workgroup (every wave computes all of them for its
// pixels); at most KMAX steps of 32 channels.
// NT2 > 0: the layer is followed by another 1 x 1 convolution with NT2 filter
// tiles that reads all of this layer's output channels (one filter group): a
// wave's finished 16-pixel tile, rounded as it is stored, is at once the pixel
// operand of the second convolution, whose output is stored as well; the
// second layer never reads the first one's output from memory.
// THREADS: 256, two workgroups to a compute unit; or 512, one workgroup whose
// eight waves share one copy of the filters, for the pairs whose two filter sets
// do not fit LDS twice.
template <bool BF, int NT, int KMAX, int NT2, int THREADS = 256, int MINB = 1>
__global__ __launch_bounds__(THREADS, MINB) void conv1x1_stream_kernel(const StreamParams p) {
  constexpr int kWaves = THREADS / 64;
  constexpr int NF = NT * 16;
  constexpr int NF2 = NT2 * 16;
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  float* bias_lds = reinterpret_cast<float*>(lds);                 // [NF]
  char* wts = lds + NF * 4;                                        // [ksteps * 4][NF][16 bytes]
  // second convolution: [NF2] bias, then [NT / 2 steps * 4][NF2][16 bytes]
  float* bias2_lds = reinterpret_cast<float*>(wts + p.w_lds_bytes);
  char* wts2 = reinterpret_cast<char*>(bias2_lds) + NF2 * 4;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, g = lane >> 4;
  const int f0 = blockIdx.y * NF;

  const __amdgpu_buffer_rsrc_t xrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x), 0, p.x_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t x2rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x2), 0, p.x2_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t wrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.w), 0, p.w_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t yrsrc =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.res), 0, p.res_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t hrsrc =
      __builtin_amdgcn_make_buffer_rsrc(p.h, 0, p.h_bytes, 0x00020000);

  // ---- filters and bias of this group -> LDS -----------------------------------------
  // straight into LDS, all loads in flight at once; slots past the group's
  // filters or the layer's channels receive zeros
  {
    const uint64_t wa = reinterpret_cast<uint64_t>(p.w);
    i32x4 wr;
    wr[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)wa);
    wr[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(wa >> 32));
    wr[2] = __builtin_amdgcn_readfirstlane((int)p.w_bytes);
    wr[3] = 0x00020000;
    const uint32_t wts_lds = (uint32_t)(uintptr_t)(LdsPtr)wts;
    const int n_slots = p.ksteps * 4 * NF;
    for (int base = wave * 64; base < n_slots; base += THREADS) {
      const int e = base + lane;
      const int chunk = e / NF, f = e - chunk * NF;
      const bool ok = e < n_slots && chunk < p.cpt && f0 + f < p.Kp;
      const uint32_t off = ok ? (uint32_t)(chunk * p.Kp + f0 + f) * 16u : kOutside;
      asm volatile(
          "s_mov_b32 m0, %0\n\t"
          "s_nop 0\n\t"
          "buffer_load_dwordx4 %1, %2, 0 offen lds"
          :
          : "s"(wts_lds + base * 16), "v"(off), "s"(wr)
          : "memory", "m0");
    }
  }
  for (int e = tid; e < NF; e += THREADS) bias_lds[e] = f0 + e < p.Kp ? p.bias[f0 + e] : 0.f;
  if constexpr (NT2 > 0) {
    const uint64_t wa = reinterpret_cast<uint64_t>(p.w2);
    i32x4 wr;
    wr[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)wa);
    wr[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(wa >> 32));
    wr[2] = __builtin_amdgcn_readfirstlane((int)p.w2_bytes);
    wr[3] = 0x00020000;
    const uint32_t wts2_lds = (uint32_t)(uintptr_t)(LdsPtr)wts2;
    constexpr int n_slots2 = (NT / 2) * 4 * NF2;
    for (int base = wave * 64; base < n_slots2; base += THREADS) {
      const int e = base + lane;
      const int chunk = e / NF2, f = e - chunk * NF2;
      const bool ok = e < n_slots2 && chunk < p.cpt2 && f < p.Kp2;
      const uint32_t off = ok ? (uint32_t)(chunk * p.Kp2 + f) * 16u : kOutside;
      asm volatile(
          "s_mov_b32 m0, %0\n\t"
          "s_nop 0\n\t"
          "buffer_load_dwordx4 %1, %2, 0 offen lds"
          :
          : "s"(wts2_lds + base * 16), "v"(off), "s"(wr)
          : "memory", "m0");
    }
    for (int e = tid; e < NF2; e += THREADS) bias2_lds[e] = e < p.Kp2 ? p.bias2[e] : 0.f;
  }

  // ---- this wave's tiles -------------------------------------------------------------
  const int n_waves = gridDim.x * kWaves;
  int tile = blockIdx.x * kWaves + wave;
  uint4 bn[KMAX] = {};
  static_assert(NT % 2 == 0, "filter tiles are handled in pairs");
  constexpr int NP = NT / 2;
  u32x4 rvn[NP] = {};
  const int k_pair = (g & 1) * 16 + (g >> 1) * 8;   // channel of this lane's 16 bytes in a tile pair
  uint32_t yoff_n = kOutside, hoff_n = kOutside;
  // The eight-wave variant keeps the pixel fragments of TWO tiles in flight per wave (the pairs
  // it serves read few bytes per pixel, and one tile per wave in flight leaves the memory
  // system short of requests: 2.7 TB/s measured).  It has no shortcut (its launcher refuses
  // one): the registers that would hold shortcut values hold the second tile.
  constexpr bool kDeep = THREADS == 512;
  // A pair built for two workgroups per compute unit has no registers for the next tile's
  // shortcut: it asks for a tile's shortcut when it starts the tile (eight waves hide the wait).
  constexpr bool kLateRes = MINB == 2 && NT2 > 0 && !kDeep;
  const bool has_res = !kDeep && p.res != nullptr;
  uint4 bn2[kDeep ? KMAX : 1] = {};
  uint32_t yoff_n2 = kOutside, hoff_n2 = kOutside;
  auto fetch_pixels = [&](int t, uint4* bdst, uint32_t& yo, uint32_t& ho, uint32_t& ro) {
    const int m = t * 16 + li;
    uint32_t xo = kOutside, xo2 = kOutside;
    ro = kOutside;
    yo = kOutside;
    ho = kOutside;
    if (m < p.M) {
      yo = (uint32_t)m * (uint32_t)(p.ycs * 2);
      ho = (uint32_t)m * (uint32_t)(p.hcs * 2);
      if (p.plain) {
        xo = (uint32_t)m * (uint32_t)(p.xcs * 2);
        ro = (uint32_t)m * (uint32_t)(p.rcs * 2);
      }
      if (!p.plain || p.x2) {
        const int n = m / p.PQ, rem = m - n * p.PQ;
        const int pp = rem / p.Q, qq = rem - pp * p.Q;
        if (!p.plain) {
          xo = (uint32_t)(((n * p.H + pp * p.stride) * p.W + qq * p.stride) * p.xcs) * 2u;
          ro = (uint32_t)(((n * p.rH + pp * p.rss) * p.rW + qq * p.rss) * p.rcs) * 2u;
        }
        xo2 = (uint32_t)(((n * p.H2 + pp * p.stride2) * p.W2 + qq * p.stride2) * p.xcs2) * 2u;
      }
    }
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      if (k < p.ksteps) {
        const int chunk = k * 4 + g;
        if (k * 4 < p.split) {   // a whole step comes from one tensor
          const uint32_t off = chunk * 8 < p.xcs ? xo + (uint32_t)chunk * 16u : kOutside;
          bdst[k] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(xrsrc, off, 0, 0));
        } else {
          const int c2 = chunk - p.split;
          const uint32_t off = c2 * 8 < p.xcs2 ? xo2 + (uint32_t)c2 * 16u : kOutside;
          bdst[k] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(x2rsrc, off, 0, 0));
        }
      }
    }
  };
  auto fetch_shortcut = [&](uint32_t ro) {
    if (has_res) {
#pragma unroll
      for (int pr = 0; pr < NP; ++pr) {
        const int rc = f0 + pr * 32 + k_pair - p.roff;
        const uint32_t off = (rc >= 0 && rc < p.rcs) ? ro + (uint32_t)rc * 2u : kOutside;
        rvn[pr] = __builtin_amdgcn_raw_buffer_load_b128(rrsrc, off, 0, 0);
      }
    }
  };
  uint32_t ro_n = kOutside, ro_n2 = kOutside;
  if (tile < p.n_tiles) {   // in flight while the filters arrive
    fetch_pixels(tile, bn, yoff_n, hoff_n, ro_n);
    if constexpr (!kLateRes) fetch_shortcut(ro_n);
    if constexpr (kDeep)
      if (tile + n_waves < p.n_tiles) fetch_pixels(tile + n_waves, bn2, yoff_n2, hoff_n2, ro_n2);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();   // filters and bias are in LDS
  const uint32_t floor2 = p.relu ? 0u : 0x80008000u;
  const char* a_lane = wts + (g * NF + li) * 16;
  // One tile: `cur` holds its pixel fragments (asked for one or two tiles ago), rvn its
  // shortcut values.  kDeep: the other register set holds the next tile's fragments, already
  // on their way; this set is refilled with the tile after that.  Otherwise this set is
  // refilled with the next tile.
  auto process = [&](uint4* cur, uint32_t& yo_cur, uint32_t& ho_cur, uint32_t& ro_cur, uint32_t ro_other) {
    uint4 b[KMAX];
    u32x4 rv[NP];
#pragma unroll
    for (int k = 0; k < KMAX; ++k) b[k] = cur[k];
    if constexpr (kLateRes) {
      fetch_shortcut(ro_cur);
    }
#pragma unroll
    for (int pr = 0; pr < NP; ++pr) rv[pr] = rvn[pr];
    const uint32_t yoff = yo_cur, hoff = ho_cur;
    if constexpr (kDeep) {
      if (tile + n_waves < p.n_tiles) fetch_shortcut(ro_other);
      if (tile + 2 * n_waves < p.n_tiles) fetch_pixels(tile + 2 * n_waves, cur, yo_cur, ho_cur, ro_cur);
    } else {
      if (tile + n_waves < p.n_tiles) {
        fetch_pixels(tile + n_waves, cur, yo_cur, ho_cur, ro_cur);
        if constexpr (!kLateRes) fetch_shortcut(ro_cur);
      }
    }

    uint4 yb[NT2 > 0 ? NP : 1];   // the finished tile as pixel fragments of the second convolution
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = *reinterpret_cast<const f32x4*>(bias_lds + t * 16 + g * 4);
#pragma unroll
    for (int k = 0; k < KMAX; ++k) {
      if (k < p.ksteps) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const uint4 a = *reinterpret_cast<const uint4*>(a_lane + (k * 4 * NF + t * 16) * 16);
          acc[t] = mfma_16x16x32<BF>(a, b[k], acc[t]);
        }
      }
    }
    // Epilogue in pairs of filter tiles exchanged between 16-lane rows: lane
    // (pixel, g) then holds channels (g >> 1) * 8 .. + 7 of tile t + (g & 1), so
    // every access is 16 bytes and a pixel's 64 bytes come from four lanes.
    auto finish = [&](const f32x4& av, uint32_t r0, uint32_t r1) {
      float v[4] = {av[0], av[1], av[2], av[3]};
      if (has_res) {
        v[0] += to_float<BF>((uint16_t)(r0 & 0xffffu));
        v[1] += to_float<BF>((uint16_t)(r0 >> 16));
        v[2] += to_float<BF>((uint16_t)(r1 & 0xffffu));
        v[3] += to_float<BF>((uint16_t)(r1 >> 16));
      }
      u32x2 o;
      o[0] = clamp_below2(pack2<BF>(v[0], v[1]), floor2);
      o[1] = clamp_below2(pack2<BF>(v[2], v[3]), floor2);
      return o;
    };
#pragma unroll
    for (int pr = 0; pr < NP; ++pr) {
      const int t = 2 * pr;
      uint32_t ra0 = 0, ra1 = 0, rb0 = 0, rb1 = 0;
      if (has_res) {
        const auto s0 = __builtin_amdgcn_permlane16_swap(rv[pr][0], rv[pr][2], false, false);
        const auto s1 = __builtin_amdgcn_permlane16_swap(rv[pr][1], rv[pr][3], false, false);
        ra0 = s0[0]; ra1 = s1[0];
        rb0 = s0[1]; rb1 = s1[1];
      }
      const u32x2 oa = finish(acc[t], ra0, ra1), ob = finish(acc[t + 1], rb0, rb1);
      const auto w0 = __builtin_amdgcn_permlane16_swap(oa[0], ob[0], false, false);
      const auto w1 = __builtin_amdgcn_permlane16_swap(oa[1], ob[1], false, false);
      const u32x4 o4 = {w0[0], w1[0], w0[1], w1[1]};
      const int k0 = f0 + pr * 32 + k_pair;
      const uint32_t off = k0 < p.ycs ? yoff + (uint32_t)k0 * 2u : kOutside;
      __builtin_amdgcn_raw_buffer_store_b128(o4, yrsrc, off, 0, 0);
      if constexpr (NT2 > 0) yb[pr] = __builtin_bit_cast(uint4, o4);
    }
    if constexpr (NT2 > 0) {
      // Pair pr of the output is step pr of the second reduction: lane (pixel, g)
      // holds channels pr * 32 + (g & 1) * 16 + (g >> 1) * 8 .. + 7, i.e. chunk
      // (g & 1) * 2 + (g >> 1) of the step, and reads the matching filter chunk.
      const char* a2_lane = wts2 + ((((g & 1) * 2 + (g >> 1)) * NF2) + li) * 16;
      f32x4 acc2[NT2];
#pragma unroll
      for (int t = 0; t < NT2; ++t)
        acc2[t] = *reinterpret_cast<const f32x4*>(bias2_lds + t * 16 + g * 4);
#pragma unroll
      for (int s2 = 0; s2 < NP; ++s2) {
        if (s2 * 4 < p.cpt2) {
#pragma unroll
          for (int t = 0; t < NT2; ++t) {
            const uint4 a2 = *reinterpret_cast<const uint4*>(a2_lane + (s2 * 4 * NF2 + t * 16) * 16);
            acc2[t] = mfma_16x16x32<BF>(a2, yb[s2], acc2[t]);
          }
        }
      }
      const uint32_t floor2b = p.relu2 ? 0u : 0x80008000u;
#pragma unroll
      for (int pr = 0; pr < NT2 / 2; ++pr) {
        u32x2 oa, ob;
        oa[0] = clamp_below2(pack2<BF>(acc2[2 * pr][0], acc2[2 * pr][1]), floor2b);
        oa[1] = clamp_below2(pack2<BF>(acc2[2 * pr][2], acc2[2 * pr][3]), floor2b);
        ob[0] = clamp_below2(pack2<BF>(acc2[2 * pr + 1][0], acc2[2 * pr + 1][1]), floor2b);
        ob[1] = clamp_below2(pack2<BF>(acc2[2 * pr + 1][2], acc2[2 * pr + 1][3]), floor2b);
        const auto w0 = __builtin_amdgcn_permlane16_swap(oa[0], ob[0], false, false);
        const auto w1 = __builtin_amdgcn_permlane16_swap(oa[1], ob[1], false, false);
        const u32x4 o4 = {w0[0], w1[0], w0[1], w1[1]};
        const int k0 = pr * 32 + k_pair;
        const uint32_t off = k0 < p.hcs ? hoff + (uint32_t)k0 * 2u : kOutside;
        __builtin_amdgcn_raw_buffer_store_b128(o4, hrsrc, off, 0, 0);
      }
    }
  };
  if constexpr (kDeep) {
    while (tile < p.n_tiles) {
      process(bn, yoff_n, hoff_n, ro_n, ro_n2);
      tile += n_waves;
      if (tile >= p.n_tiles) break;
      process(bn2, yoff_n2, hoff_n2, ro_n2, ro_n);
      tile += n_waves;
    }
  } else {
    for (; tile < p.n_tiles; tile += n_waves) process(bn, yoff_n, hoff_n, ro_n, ro_n);
  }
}

struct StreamTile {
  int NT, KMAX;
  const char* name;
};
constexpr StreamTile kStreamTiles[] = {
    {16, 2, "conv1x1s_256f"}, {16, 4, "conv1x1s_256f_c128"}, {8, 8, "conv1x1s_128f"},
    {4, 8, "conv1x1s_64f"},   {4, 16, "conv1x1s_64f_c512"},  {2, 8, "conv1x1s_32f"},
};
constexpr int kNumStreamTiles = sizeof(kStreamTiles) / sizeof(kStreamTiles[0]);

int stream_compute_units() {
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

size_t stream_lds_bytes(const StreamTile& t, int ksteps) {
  // the filter area is written by whole waves of 1 KB
  return (size_t)t.NT * 16 * 4 + round_up_sz((size_t)ksteps * 4 * t.NT * 16 * 16, 1024);
}

// The widest filter group whose filters fit; -1: the layer is not for this kernel.
int pick_stream(const Conv16Params& c) {
  if (tuning_off("conv1x1_stream")) return -1;
  if (c.S != 1 || c.nchunk != c.cpt || c.pad != 0 || (c.stride != 1 && c.stride != 2)) return -1;
  if (c.roff % 8 != 0) return -1;   // 16-byte shortcut loads
  const int ksteps = (c.cpt + 3) / 4;
  const int forced = tuning_int("stream_tile", -1);   // taken if the layer fits it
  int best = -1;
  double best_cost = 1e30;
  for (int i = 0; i < kNumStreamTiles; ++i) {
    const StreamTile& t = kStreamTiles[i];
    if (ksteps > t.KMAX || stream_lds_bytes(t, ksteps) > (size_t)kStreamLdsLimit) continue;
    if (i == forced) return i;
    // padded filter tiles, and the input is read once per group
    const int groups = (c.FT + t.NT - 1) / t.NT;
    const double cost = (double)groups * t.NT * 32.0 + (double)groups * c.cpt * 16.0 +
                        (t.KMAX - ksteps) * 0.01;
    if (cost < best_cost) {
      best_cost = cost;
      best = i;
    }
  }
  return best;
}

template <bool BF, int NT, int KMAX, int NT2 = 0, int THREADS = 256, int MINB = 1>
fupr_status launch_stream(const StreamParams& p, dim3 grid, size_t lds, hipStream_t st) {
  static std::once_flag once;
  static hipError_t status = hipSuccess;
  std::call_once(once, [] {
    status = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&conv1x1_stream_kernel<BF, NT, KMAX, NT2, THREADS, MINB>),
        hipFuncAttributeMaxDynamicSharedMemorySize,
        THREADS == 256 && NT2 <= 4 ? kStreamFusedLdsLimit : 2 * kStreamFusedLdsLimit);
  });
  if (status != hipSuccess) return FUPR_ERR_LAUNCH;
  hipLaunchKernelGGL((conv1x1_stream_kernel<BF, NT, KMAX, NT2, THREADS, MINB>), grid, dim3(THREADS), lds, st, p);
  return launch_status("conv1x1_stream_kernel");
}

template <bool BF>
fupr_status dispatch_stream(int tile, const StreamParams& p, dim3 grid, size_t lds,
                            hipStream_t st) {
  // Compiled for two workgroups per compute unit (at most 256 registers): the MFMAs keep
  // their accumulators in ordinary registers, without the copies to and from the
  // accumulation registers that the one-workgroup build spends per tile, and eight waves
  // keep loads in flight (config 4: 2800 -> 2736 us).
  if (tuning_int("stream_blocks", 2) >= 2) {
    switch (tile) {
      case 0: return launch_stream<BF, 16, 2, 0, 256, 2>(p, grid, lds, st);
      case 1: return launch_stream<BF, 16, 4, 0, 256, 2>(p, grid, lds, st);
      case 2: return launch_stream<BF, 8, 8, 0, 256, 2>(p, grid, lds, st);
      case 3: return launch_stream<BF, 4, 8, 0, 256, 2>(p, grid, lds, st);
      case 4: return launch_stream<BF, 4, 16, 0, 256, 2>(p, grid, lds, st);
      default: return launch_stream<BF, 2, 8, 0, 256, 2>(p, grid, lds, st);
    }
  }
  switch (tile) {
    case 0: return launch_stream<BF, 16, 2>(p, grid, lds, st);
    case 1: return launch_stream<BF, 16, 4>(p, grid, lds, st);
    case 2: return launch_stream<BF, 8, 8>(p, grid, lds, st);
    case 3: return launch_stream<BF, 4, 8>(p, grid, lds, st);
    case 4: return launch_stream<BF, 4, 16>(p, grid, lds, st);
    default: return launch_stream<BF, 2, 8>(p, grid, lds, st);
  }
}

}  // namespace

bool conv1x1_stream_applies(const Conv16Params& c) { return pick_stream(c) >= 0; }

const char* conv1x1_stream_name(const Conv16Params& c) {
  const int t = pick_stream(c);
  return t < 0 ? "conv1x1s" : kStreamTiles[t].name;
}

namespace {

// Everything but the second convolution's fields; false if a tensor is too large.
bool fill_stream_params(const Conv16Params& c, int N, StreamParams* out) {
  StreamParams p{};
  p.x = c.x; p.w = c.w; p.bias = c.bias; p.res = c.res; p.y = c.y;
  const uint64_t y_bytes = (uint64_t)c.M * c.ycs * 2;
  const uint64_t res_bytes = c.res ? (uint64_t)N * c.rH * c.rW * c.rcs * 2 : 0;
  if ((uint64_t)c.x_bytes >= kOutside || y_bytes >= kOutside || res_bytes >= kOutside ||
      (uint64_t)c.x2_bytes >= kOutside)
    return false;
  p.x_bytes = c.x_bytes; p.w_bytes = c.w_bytes;
  p.y_bytes = (uint32_t)y_bytes; p.res_bytes = (uint32_t)res_bytes;
  p.H = c.H; p.W = c.W; p.xcs = c.xcs;
  p.P = c.P; p.Q = c.Q; p.PQ = c.PQ; p.M = c.M; p.ycs = c.ycs;
  p.stride = c.stride;
  p.Kp = c.Kp; p.cpt = c.cpt; p.ksteps = (c.cpt + 3) / 4;
  p.rH = c.rH; p.rW = c.rW; p.rcs = c.rcs; p.rss = c.rss; p.roff = c.roff;
  p.relu = c.relu;
  p.plain = c.stride == 1 && (!c.res || (c.rss == 1 && c.rH == c.P && c.rW == c.Q));
  p.x2 = c.x2; p.x2_bytes = c.x2_bytes;
  p.split = c.x2 ? c.split : (1 << 30);
  p.H2 = c.H2; p.W2 = c.W2; p.xcs2 = c.xcs2; p.stride2 = c.stride2;
  p.n_tiles = (c.M + 15) / 16;
  *out = p;
  return true;
}

// Which 16-tile variant (2 or 4 steps) and how many second-layer filter tiles a
// fused pair needs; false if the pair is not for the fused kernel.  A pair whose
// filters fit LDS only once runs as one workgroup of eight waves per compute unit.
bool plan_fused(const Conv16Params& c1, const Conv16Params& c2, int* kmax, int* nt2, size_t* lds) {
  if (tuning_off("conv1x1_fuse")) return false;
  const int t = pick_stream(c1);
  if (t < 0 || kStreamTiles[t].NT != 16 || c1.FT > 16 || c1.stride != 1) return false;
  if (c2.S != 1 || c2.nchunk != c2.cpt || c2.pad != 0 || c2.stride != 1 || c2.res) return false;
  if (c2.cpt * 8 != c1.ycs || c2.cpt > 32 || c2.FT > 8) return false;   // reads all of y's channels
  if (c2.FT * 16 > tuning_int("pair_filters", 128)) return false;
  if (c2.H != c1.P || c2.W != c1.Q) return false;
  *kmax = kStreamTiles[t].KMAX;
  *nt2 = 2 * ((std::max(c2.FT, 1) + 1) / 2);
  const int ksteps = (c1.cpt + 3) / 4;
  *lds = stream_lds_bytes(kStreamTiles[t], ksteps) + (size_t)*nt2 * 16 * 4 +
         (size_t)8 * 4 * *nt2 * 16 * 16;
  // 65 - 128 second filters: four waves, one workgroup per compute unit (the
  // sixteen-tile variants take more than half of a SIMD's registers per wave
  // anyway), all of LDS
  if (*nt2 > 4) return *lds <= 2 * (size_t)kStreamFusedLdsLimit;
  // (the eight-wave variant has no shortcut in its epilogue)
  return *lds <= (size_t)kStreamFusedLdsLimit ||
         (*kmax == 4 && !c1.res && *lds <= 2 * (size_t)kStreamFusedLdsLimit);
}

}  // namespace

fupr_status launch_conv1x1_stream(const Conv16Params& c, int N, bool bf16, void* stream) {
  const int t = pick_stream(c);
  if (t < 0) return FUPR_ERR_LIMIT;
  const StreamTile& tile = kStreamTiles[t];
  StreamParams p;
  if (!fill_stream_params(c, N, &p)) return FUPR_ERR_LIMIT;
  const int groups = (c.FT + tile.NT - 1) / tile.NT;
  // persistent workgroups, two per compute unit over all filter groups
  const int per_group = std::max(1, 2 * stream_compute_units() / groups);
  const int gx = std::min((p.n_tiles + 3) / 4, per_group);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)gx, (unsigned)groups);
  const size_t lds = stream_lds_bytes(tile, p.ksteps);
  return bf16 ? dispatch_stream<true>(t, p, grid, lds, st)
              : dispatch_stream<false>(t, p, grid, lds, st);
}

bool conv1x1_fused_pair_applies(const Conv16Params& c1, const Conv16Params& c2) {
  int kmax, nt2;
  size_t lds;
  return plan_fused(c1, c2, &kmax, &nt2, &lds);
}

fupr_status launch_conv1x1_fused_pair(const Conv16Params& c1, const Conv16Params& c2, int N,
                                      bool bf16, void* stream) {
  int kmax, nt2;
  size_t lds;
  if (!plan_fused(c1, c2, &kmax, &nt2, &lds)) return FUPR_ERR_LIMIT;
  StreamParams p;
  if (!fill_stream_params(c1, N, &p)) return FUPR_ERR_LIMIT;
  const uint64_t h_bytes = (uint64_t)c2.M * c2.ycs * 2;
  if (h_bytes >= kOutside) return FUPR_ERR_LIMIT;
  p.w2 = c2.w; p.bias2 = c2.bias; p.h = c2.y;
  p.w2_bytes = c2.w_bytes; p.h_bytes = (uint32_t)h_bytes;
  p.Kp2 = c2.Kp; p.cpt2 = c2.cpt; p.hcs = c2.ycs; p.relu2 = c2.relu;
  p.w_lds_bytes = (int)round_up_sz((size_t)p.ksteps * 4 * 16 * 16 * 16, 1024);
  // eight waves share the filters and keep two tiles in flight each: needed when the filters
  // fit LDS once only, and faster whenever there is no shortcut to read (few bytes per pixel)
  const bool wide = nt2 <= 4 && (lds > (size_t)kStreamFusedLdsLimit || (kmax == 4 && !c1.res));
  const int gx = wide ? std::min((p.n_tiles + 7) / 8, stream_compute_units())
                      : std::min((p.n_tiles + 3) / 4,
                                 (lds > (size_t)kStreamFusedLdsLimit ? 1 : 2) * stream_compute_units());
  const dim3 grid((unsigned)gx, 1u);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int key = (bf16 ? 100 : 0) + kmax * 10 + nt2 + (wide ? 1000 : 0);
  // The pairs with up to 64 second filters whose filters fit LDS twice are built for two
  // workgroups per compute unit as well (config 3: 884 -> 864 us; config 4 unchanged).
  if (!wide && tuning_int("stream_blocks", 2) >= 2 && lds <= (size_t)kStreamFusedLdsLimit) {
    switch (key) {
      case 122: return launch_stream<true, 16, 2, 2, 256, 2>(p, grid, lds, st);
      case 124: return launch_stream<true, 16, 2, 4, 256, 2>(p, grid, lds, st);
      case 142: return launch_stream<true, 16, 4, 2, 256, 2>(p, grid, lds, st);
      case 144: return launch_stream<true, 16, 4, 4, 256, 2>(p, grid, lds, st);
      case 22: return launch_stream<false, 16, 2, 2, 256, 2>(p, grid, lds, st);
      case 24: return launch_stream<false, 16, 2, 4, 256, 2>(p, grid, lds, st);
      case 42: return launch_stream<false, 16, 4, 2, 256, 2>(p, grid, lds, st);
      case 44: return launch_stream<false, 16, 4, 4, 256, 2>(p, grid, lds, st);
      default: break;
    }
  }
  switch (key) {
    case 122: return launch_stream<true, 16, 2, 2>(p, grid, lds, st);
    case 124: return launch_stream<true, 16, 2, 4>(p, grid, lds, st);
    case 142: return launch_stream<true, 16, 4, 2>(p, grid, lds, st);
    case 144: return launch_stream<true, 16, 4, 4>(p, grid, lds, st);
    case 126: return launch_stream<true, 16, 2, 6>(p, grid, lds, st);
    case 128: return launch_stream<true, 16, 2, 8>(p, grid, lds, st);
    case 146: return launch_stream<true, 16, 4, 6>(p, grid, lds, st);
    case 148: return launch_stream<true, 16, 4, 8>(p, grid, lds, st);
    case 26: return launch_stream<false, 16, 2, 6>(p, grid, lds, st);
    case 28: return launch_stream<false, 16, 2, 8>(p, grid, lds, st);
    case 46: return launch_stream<false, 16, 4, 6>(p, grid, lds, st);
    case 48: return launch_stream<false, 16, 4, 8>(p, grid, lds, st);
    case 22: return launch_stream<false, 16, 2, 2>(p, grid, lds, st);
    case 24: return launch_stream<false, 16, 2, 4>(p, grid, lds, st);
    case 42: return launch_stream<false, 16, 4, 2>(p, grid, lds, st);
    case 44: return launch_stream<false, 16, 4, 4>(p, grid, lds, st);
    case 1142: return launch_stream<true, 16, 4, 2, 512>(p, grid, lds, st);
    case 1144: return launch_stream<true, 16, 4, 4, 512>(p, grid, lds, st);
    case 1042: return launch_stream<false, 16, 4, 2, 512>(p, grid, lds, st);
    case 1044: return launch_stream<false, 16, 4, 4, 512>(p, grid, lds, st);
    default: return FUPR_ERR_LIMIT;
  }
}

}  // namespace fupr
