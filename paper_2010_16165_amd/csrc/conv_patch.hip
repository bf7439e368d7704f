// 3 x 3 convolution (pad 1, stride 1 or 2) of one layer with the input patch of
// a workgroup staged in LDS (Sec. III, Sec. IV-B-1: operator k x c x 3 x 3; the
// epilogue applies what Sec. VI-B-3 merges and the block's addition and ReLU).
//
// The tiled kernel loads every pixel fragment from global memory once per tap
// with its own range check; its instruction stream (7.6 vector + 3.3 scalar
// instructions per MFMA on the ResNet-18 layers) bounds it, not the MFMAs.
// Here a workgroup owns a strip of consecutive output pixels of one image
// and a group of filters, and walks the input channels 32 at a time:
//   * the strip's input rows, full width plus a column of zeros on each side,
//     go global -> LDS for those 32 channels (two planes of 16 channels, pixel
//     stride 32 bytes: the stride at which 16-byte-per-lane reads run at full
//     rate), rows outside the image are zeros written once;
//   * the 9 x 4 weight chunks of the filter group go global -> LDS;
//   * every tap is then one MFMA 16x16x32 step whose pixel fragment is an LDS
//     read at (pixel base + row offset) + immediate column offset: 3 address
//     additions per pixel tile per 9 steps, no range checks.
// Two workgroups share a compute unit, so one computes while the other stages.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstdlib>
#include <mutex>

#include "conv16.h"
#include "device_utils.h"
#include "fupr.h"
#include "layout.h"

namespace fupr {
namespace {

constexpr int kPatchThreads = 256;
constexpr int kPatchWaves = 4;
constexpr int kMaxPatchLoads = 12;   // 16-byte slots of the patch per thread and stage

struct PatchParams {
  const uint16_t* x;
  const uint16_t* w;     // [nchunk_pad][Kp][8]
  const float* bias;
  const uint16_t* res;
  uint16_t* y;
  int H, W, xcs;
  int P, Q, PQ, ycs;
  int stride;
  int Kp, cpt, n_stages;
  int rH, rW, rcs, rss, roff;
  int relu;
  int strips;            // per image
  int PR, Wh;            // patch rows; patch columns = W + 2
  int plane_bytes;       // PR * Wh * 32
  int patch_slots;       // 2 planes * PR * Wh * 2 halves
  int n_loads;           // ceil(patch_slots / 256)
  uint32_t magicQ, magicWh, magicPR;
};

__device__ __forceinline__ int div_by(int v, uint32_t magic) {
  return magic ? (int)__umulhi((uint32_t)v, magic) : v;
}

// lane i moves 16 bytes from src_base + lane_offset to the i-th slot after lds_base
__device__ __forceinline__ void load_to_lds(const void* src_base, uint32_t lane_offset,
                                            uint32_t lds_base) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_base), "v"(lane_offset), "s"(src_base)
      : "memory", "m0");
}

typedef void __attribute__((address_space(3)))* LdsPtr;
typedef short short2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t clamp_below(uint32_t v, uint32_t floor2) {
  const short2_t a = __builtin_bit_cast(short2_t, v), f = __builtin_bit_cast(short2_t, floor2);
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, f));
}

// MT pixel tiles x NT filter tiles of 16 x 16 per wave; the 4 waves of a
// workgroup sit side by side along the pixels: 64 * MT pixels x 16 * NT filters.
template <bool BF, int MT, int NT>
__global__ __launch_bounds__(kPatchThreads) void conv_patch_kernel(const PatchParams p) {
  constexpr int NF = NT * 16;
  constexpr int BM = kPatchWaves * MT * 16;
  constexpr int kWeightSlots = 36 * NF;                              // 9 taps x 4 chunks x NF filters
  constexpr int kWeightLoads = (kWeightSlots + kPatchThreads - 1) / kPatchThreads;
  constexpr int kWStep = 4 * NF * 16;                                // bytes of weights per tap
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  char* wts = lds;                                                   // [36][NF][16 bytes]
  char* patch = lds + kWeightSlots * 16;                             // [2][PR][Wh][32 bytes]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 15, g = lane >> 4;
  const int n = blockIdx.x / p.strips, strip = blockIdx.x - n * p.strips;
  const int f0 = blockIdx.y * NF;
  const int m0 = strip * BM;                          // first output pixel of the strip
  const int p_lo = div_by(m0, p.magicQ);              // its output row
  const int in_row0 = p_lo * p.stride - 1;            // image row of patch row 0

  // ---- what this thread stages of the patch: fixed for all channel stages ----
  int goff[kMaxPatchLoads];      // element offset in x of the slot's 8 channels at c0 = 0; -1: none
  int chunk_of[kMaxPatchLoads];  // which of the stage's four 8-channel chunks
#pragma unroll
  for (int i = 0; i < kMaxPatchLoads; ++i) {
    goff[i] = -1;
    chunk_of[i] = 0;
    if (i < p.n_loads) {
      const int s = (i * kPatchWaves + wave) * 64 + lane;
      const int half = s & 1, t = s >> 1;
      const int t2 = div_by(t, p.magicWh), col = t - t2 * p.Wh;
      const int plane = div_by(t2, p.magicPR), row = t2 - plane * p.PR;
      const int ih = in_row0 + row, iw = col - 1;
      chunk_of[i] = plane * 2 + half;
      if (s < p.patch_slots) {
        if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
          goff[i] = ((n * p.H + ih) * p.W + iw) * p.xcs + plane * 16 + half * 8;
        else   // outside the image: zeros, written once
          *reinterpret_cast<uint4*>(patch + s * 16) = uint4{0u, 0u, 0u, 0u};
      }
    }
  }

  // ---- this lane's pixels ------------------------------------------------------
  const int row_bytes = p.Wh * 32;
  int m[MT], rin[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    m[mt] = m0 + (wave * MT + mt) * 16 + li;
    const int mc = min(m[mt], p.PQ - 1);
    const int pp = div_by(mc, p.magicQ), qq = mc - pp * p.Q;
    rin[mt] = ((pp - p_lo) * p.stride * p.Wh + qq * p.stride) * 32 + (g >> 1) * p.plane_bytes +
              (g & 1) * 16;
  }
  const int a_lane = g * (NF * 16) + li * 16;

  f32x4 acc[MT][NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int k0 = min(f0 + t * 16, p.Kp - 16) + g * 4;
    const f32x4 b4 = *reinterpret_cast<const f32x4*>(p.bias + k0);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt][t] = b4;
  }

  const uint32_t lane_off16 = lane * 16;
  const uint32_t patch_lds = (uint32_t)(uintptr_t)(LdsPtr)patch;
  const uint32_t wts_lds = (uint32_t)(uintptr_t)(LdsPtr)wts;
  const int xchunks = p.xcs >> 3;

  for (int stage = 0; stage < p.n_stages; ++stage) {
    const int c0 = stage * 32;
    if (stage > 0) __syncthreads();   // everybody has read the previous stage
    // weights: row = tap * 4 + chunk of the stage, NF filters of 16 bytes each
#pragma unroll
    for (int i = 0; i < kWeightLoads; ++i) {
      const int sbase = (i * kPatchWaves + wave) * 64, s = sbase + lane;
      if (s < kWeightSlots) {
        const int row = s / NF, f = s - row * NF;
        const int tap = row >> 2, cc = (c0 >> 3) + (row & 3);
        // a chunk past the last one repeats the tap's first (finite; the patch is zero there)
        const int chunk = tap * p.cpt + (cc < p.cpt ? cc : 0);
        const int filt = min(f0 + f, p.Kp - 1);
        load_to_lds(p.w, (uint32_t)(chunk * p.Kp + filt) * 16u, wts_lds + sbase * 16);
      }
    }
    // patch
#pragma unroll
    for (int i = 0; i < kMaxPatchLoads; ++i) {
      if (i < p.n_loads && goff[i] >= 0) {
        const int sbase = (i * kPatchWaves + wave) * 64, s = sbase + lane;
        if ((c0 >> 3) + chunk_of[i] < xchunks)
          load_to_lds(p.x, (uint32_t)(goff[i] + c0) * 2u, patch_lds + sbase * 16);
        else   // past the last channel: zeros
          *reinterpret_cast<uint4*>(patch + s * 16) = uint4{0u, 0u, 0u, 0u};
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // 9 taps = 9 MFMA steps over these 32 channels; the operands of a step are
    // read while the step before it is multiplied
    int brow[3][MT];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) brow[r][mt] = rin[mt] + r * row_bytes;
    uint4 a[2][NT], b[2][MT];
    auto operands = [&](int tap, uint4* av, uint4* bv) {
      const int r = tap / 3, sx = tap - r * 3;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        bv[mt] = *reinterpret_cast<const uint4*>(patch + brow[r][mt] + sx * 32);
#pragma unroll
      for (int t = 0; t < NT; ++t)
        av[t] = *reinterpret_cast<const uint4*>(wts + a_lane + tap * kWStep + t * 256);
    };
    operands(0, a[0], b[0]);
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      if (tap + 1 < 9) operands(tap + 1, a[(tap + 1) & 1], b[(tap + 1) & 1]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[mt][t] = mfma_16x16x32<BF>(a[tap & 1][t], b[tap & 1][mt], acc[mt][t]);
    }
  }

  // ---- epilogue: shortcut, ReLU, one rounding ------------------------------------
  const uint32_t floor2 = p.relu ? 0u : 0x80008000u;
  const int m_end = min(m0 + BM, p.PQ);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (m[mt] >= m_end) continue;
    const int pp = div_by(m[mt], p.magicQ), qq = m[mt] - pp * p.Q;
    const size_t ypix = ((size_t)n * p.PQ + m[mt]) * p.ycs;
    const size_t rpix =
        p.res ? (((size_t)n * p.rH + (size_t)pp * p.rss) * p.rW + (size_t)qq * p.rss) * p.rcs : 0;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int k0 = f0 + t * 16 + g * 4;
      if (k0 >= p.ycs) continue;
      float v[4] = {acc[mt][t][0], acc[mt][t][1], acc[mt][t][2], acc[mt][t][3]};
      if (p.res) {
        const int rc = k0 - p.roff;
        if (rc >= 0 && rc < p.rcs) {
          const uint2 rv = *reinterpret_cast<const uint2*>(p.res + rpix + rc);
          v[0] += to_float<BF>((uint16_t)(rv.x & 0xffffu));
          v[1] += to_float<BF>((uint16_t)(rv.x >> 16));
          v[2] += to_float<BF>((uint16_t)(rv.y & 0xffffu));
          v[3] += to_float<BF>((uint16_t)(rv.y >> 16));
        }
      }
      uint2 o;
      o.x = clamp_below(pack2<BF>(v[0], v[1]), floor2);
      o.y = clamp_below(pack2<BF>(v[2], v[3]), floor2);
      *reinterpret_cast<uint2*>(p.y + ypix + k0) = o;
    }
  }
}

uint32_t reciprocal(int d) { return d == 1 ? 0u : 0xffffffffu / (uint32_t)d + 1u; }

struct PatchTile {
  int MT, NT;
};

// Filters per workgroup: 64, or 48 / 32 when that pads less.
int choose_patch_nt(int FT) {
  const int waste4 = (FT + 3) / 4 * 4 - FT, waste3 = (FT + 2) / 3 * 3 - FT;
  return FT <= 2 ? 2 : (waste3 < waste4 ? 3 : 4);
}

// Fills the parameters that depend on the tile; false if the layer does not fit.
bool plan_patch(const Conv16Params& c, int N, const PatchTile& tile, PatchParams* out,
                size_t* lds_bytes, dim3* grid) {
  PatchParams p{};
  const int BM = kPatchWaves * tile.MT * 16, NF = tile.NT * 16;
  p.x = c.x; p.w = c.w; p.bias = c.bias; p.res = c.res; p.y = c.y;
  p.H = c.H; p.W = c.W; p.xcs = c.xcs;
  p.P = c.P; p.Q = c.Q; p.PQ = c.PQ; p.ycs = c.ycs;
  p.stride = c.stride;
  p.Kp = c.Kp; p.cpt = c.cpt; p.n_stages = (c.cpt + 3) / 4;
  p.rH = c.rH; p.rW = c.rW; p.rcs = c.rcs; p.rss = c.rss; p.roff = c.roff;
  p.relu = c.relu;
  p.strips = (c.PQ + BM - 1) / BM;
  const int rows_out = std::min(c.P, (BM - 1 + c.Q - 1) / c.Q + 1);   // rows a strip can touch
  p.PR = (rows_out - 1) * c.stride + 3;
  p.Wh = c.W + 2;
  p.plane_bytes = p.PR * p.Wh * 32;
  p.patch_slots = 2 * p.PR * p.Wh * 2;
  p.n_loads = (p.patch_slots + kPatchThreads - 1) / kPatchThreads;
  if (p.n_loads > kMaxPatchLoads) return false;
  p.magicQ = reciprocal(c.Q);
  p.magicWh = reciprocal(p.Wh);
  p.magicPR = reciprocal(p.PR);
  if ((int64_t)p.patch_slots >= 65536 || c.PQ >= 65536) return false;   // reciprocal range
  *lds_bytes = (size_t)36 * NF * 16 + (size_t)2 * p.plane_bytes;
  if (*lds_bytes > 80 * 1024) return false;   // two workgroups per compute unit
  const int64_t gx = (int64_t)N * p.strips;
  if (gx >= (int64_t(1) << 31)) return false;
  *grid = dim3((unsigned)gx, (unsigned)((c.Kp + NF - 1) / NF));
  *out = p;
  return true;
}

template <bool BF, int MT, int NT>
fupr_status launch_patch(const PatchParams& p, size_t lds_bytes, dim3 grid, hipStream_t st) {
  static std::once_flag once;
  static hipError_t status = hipSuccess;
  std::call_once(once, [] {
    status = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_patch_kernel<BF, MT, NT>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
  });
  if (status != hipSuccess) return FUPR_ERR_LAUNCH;
  hipLaunchKernelGGL((conv_patch_kernel<BF, MT, NT>), grid, dim3(kPatchThreads), lds_bytes, st, p);
  return launch_status("conv_patch_kernel");
}

template <bool BF>
fupr_status dispatch_patch(const PatchTile& t, const PatchParams& p, size_t lds, dim3 grid,
                           hipStream_t st) {
  switch (t.MT * 8 + t.NT) {
    case 4 * 8 + 4: return launch_patch<BF, 4, 4>(p, lds, grid, st);
    case 4 * 8 + 3: return launch_patch<BF, 4, 3>(p, lds, grid, st);
    case 4 * 8 + 2: return launch_patch<BF, 4, 2>(p, lds, grid, st);
    case 2 * 8 + 4: return launch_patch<BF, 2, 4>(p, lds, grid, st);
    case 2 * 8 + 3: return launch_patch<BF, 2, 3>(p, lds, grid, st);
    case 2 * 8 + 2: return launch_patch<BF, 2, 2>(p, lds, grid, st);
    case 1 * 8 + 4: return launch_patch<BF, 1, 4>(p, lds, grid, st);
    case 1 * 8 + 3: return launch_patch<BF, 1, 3>(p, lds, grid, st);
    default: return launch_patch<BF, 1, 2>(p, lds, grid, st);
  }
}

bool patch_disabled() {
  const char* e = std::getenv("FUPR_CONV_PATCH");
  return e && e[0] == '0';
}

// Pixels per workgroup: 256 / 128 / 64, the largest that the image's pixel
// count (a strip never spans two images) and LDS allow.
bool pick_patch(const Conv16Params& c, int N, PatchTile* tile, PatchParams* p, size_t* lds,
                dim3* grid) {
  tile->NT = choose_patch_nt(c.FT);
  for (int mt = c.PQ > 128 ? 4 : (c.PQ > 64 ? 2 : 1); mt >= 1; mt /= 2) {
    tile->MT = mt;
    if (plan_patch(c, N, *tile, p, lds, grid)) return true;
  }
  return false;
}

}  // namespace

bool conv_patch_applies(const Conv16Params& c) {
  if (patch_disabled()) return false;
  if (c.S != 3 || c.nchunk != 9 * c.cpt || c.pad != 1 || (c.stride != 1 && c.stride != 2))
    return false;
  if (c.cpt < 2) return false;   // fewer than 16 channels: nothing to reuse
  PatchTile tile;
  PatchParams p;
  size_t lds;
  dim3 grid;
  return pick_patch(c, 1, &tile, &p, &lds, &grid);
}

const char* conv_patch_name(const Conv16Params& c) {
  static const char* names[3][3] = {{"conv3x3p_64x32", "conv3x3p_64x48", "conv3x3p_64x64"},
                                    {"conv3x3p_128x32", "conv3x3p_128x48", "conv3x3p_128x64"},
                                    {"conv3x3p_256x32", "conv3x3p_256x48", "conv3x3p_256x64"}};
  PatchTile t;
  PatchParams p;
  size_t lds;
  dim3 grid;
  if (!pick_patch(c, 1, &t, &p, &lds, &grid)) return "conv3x3p";
  return names[t.MT == 4 ? 2 : t.MT == 2 ? 1 : 0][t.NT - 2];
}

fupr_status launch_conv_patch(const Conv16Params& c, int N, bool bf16, void* stream) {
  PatchTile tile;
  PatchParams p;
  size_t lds;
  dim3 grid;
  if (!pick_patch(c, N, &tile, &p, &lds, &grid)) return FUPR_ERR_LIMIT;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  return bf16 ? dispatch_patch<true>(tile, p, lds, grid, st)
              : dispatch_patch<false>(tile, p, lds, grid, st);
}

}  // namespace fupr
