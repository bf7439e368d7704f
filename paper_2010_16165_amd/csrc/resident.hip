// A whole small-image network in ONE kernel: one workgroup per image, every
// activation tensor of that image AND the current layer's parameters resident
// in LDS, layers walked from a table.
//
// At CIFAR sizes (Table II, 32x32 inputs) each per-layer kernel runs for a few
// microseconds and the forward pass is bound by launches and by activations
// bouncing through L2; here an image's activations never leave the compute unit
// between the input read and the logits write.  What the paper removes by
// folding non-parametric operators into convolutions ("Sys.", "BN", "Add"
// columns of Table VI) is removed here one level further: the operator
// boundaries themselves.
//
// Per layer: the next layer's parameter blob and tap table are on their way from
// global memory into LDS WHILE the current layer is computed, so no
// global-memory latency sits on the layer chain; both MFMA operands of the
// current layer (filters = A, pixels = B) come from LDS.
// A work item is MT pixel tiles x NT filter tiles of 16 x 16, so every LDS
// fragment feeds several MFMAs.
//
// The instruction stream around the MFMAs is what bounds a network this small,
// so it is kept short: the accumulator starts from the bias, and the shortcut is
// added by one more MFMA step whose filter operand is a one-hot (identity)
// fragment built in registers — the epilogue is ReLU, one rounding and one LDS
// store.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "device_utils.h"
#include "fupr.h"
#include "layout.h"

namespace fupr {
namespace {

constexpr int kWaves = kResThreads / 64;

// floor(v / d) for v < 2^16 from the host's reciprocal of d (0 stands for d = 1).
__device__ __forceinline__ int div_magic(int v, uint32_t magic) {
  return magic ? (int)__umulhi((uint32_t)v, magic) : v;
}

// Zeroes the halo ring (hp pixels wide) around a P x Q tensor whose interior
// starts at byte offset org; Wh = Q + 2*hp pixels per row, ps2 bytes per pixel,
// chunks 16-byte units per pixel that hold channels.
__device__ __forceinline__ void zero_halo(char* act, int org, int P, int Q, int Wh, int ps2,
                                          int chunks, int hp, int tid) {
  const int raw = org - hp * (Wh + 1) * ps2;
  const int top_bottom = 2 * hp * Wh;
  const int total = (top_bottom + 2 * hp * P) * chunks;
  for (int i = tid; i < total; i += kResThreads) {
    const int px = i / chunks, ch = i - px * chunks;
    int row, col;
    if (px < top_bottom) {
      const int rr = px / Wh;
      col = px - rr * Wh;
      row = rr < hp ? rr : P + rr;
    } else {
      const int q = px - top_bottom;
      const int rr = q / (2 * hp), cc = q - rr * 2 * hp;
      row = hp + rr;
      col = cc < hp ? cc : Q + cc;
    }
    *reinterpret_cast<uint4*>(act + raw + (row * Wh + col) * ps2 + ch * 16) = uint4{0u, 0u, 0u, 0u};
  }
}

// The filter fragment of the shortcut step for filter tile ft: row i (= filter
// ft*16 + i) has a single 1.0 at reduction index i, so the MFMA adds shortcut
// channel ft*16 + i to that filter's accumulator; rows beyond the shortcut's
// channel count stay zero (a shortcut with fewer channels than the block
// output is the zero-padded kind).
template <bool BF>
__device__ __forceinline__ uint4 identity_fragment(int ft, int res_cs, int li, int g) {
  const uint32_t one = BF ? 0x3f80u : 0x3c00u;
  const bool on = g == (li >> 3) && ft * 16 + li < res_cs;
  const uint32_t v = on ? one << ((li & 1) * 16) : 0u;
  const int j = (li & 7) >> 1;
  return uint4{j == 0 ? v : 0u, j == 1 ? v : 0u, j == 2 ? v : 0u, j == 3 ? v : 0u};
}

// All work items of one conv layer that fall to this wave.  LAST: the layer
// writes the network output to global memory instead of LDS.
//
// Every activation tensor in LDS carries a ring of zero pixels as wide as the
// largest padding of any convolution, so a tap never needs a bounds check: the
// K loop is one table read, MT + 1 address additions, MT + NT LDS reads and
// MT * NT MFMAs per step.  D steps of operands are kept in flight (ring of
// register buffers, loop unrolled by D).
template <bool BF, int MT, int NT, bool LAST>
__device__ __forceinline__ void conv_items(const ResLayer& L, const ResParams& p, char* act,
                                           int n, int lane, int wave) {
  constexpr int D = (MT + NT <= 3) ? 4 : (MT + NT == 4 ? 3 : 2);
  const int li = lane & 15, g = lane >> 4;
  const int nsteps = L.nsteps, FT = L.FT, M = L.M, Q = L.Q;
  const bool relu = (L.flags & kResRelu) != 0, has_res = L.res_org >= 0;
  const int ycs = LAST ? p.y_cs : L.cs_out;
  const int wstep = L.wstep;
  const int a_lane = L.wts_off + g * (wstep >> 2) + li * 16;
  const float* bias = reinterpret_cast<const float*>(act + L.w_off);
  const int* tabg = reinterpret_cast<const int*>(act + L.tab_off) + g;
  const int n_items = L.n_items, n_fgroups = L.n_fgroups;

  for (int item = wave; item < n_items; item += kWaves) {
    const int pg = div_magic(item, L.magicF);
    const int ft0 = (item - pg * n_fgroups) * NT;
    // filter tiles past the last one repeat it (computed, not stored)
    int ft[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) ft[t] = min(ft0 + t, FT - 1);

    // table entries of the first steps and the bias are requested first: their
    // latency passes while the pixel addresses are worked out
    int e0[D];
#pragma unroll
    for (int d = 0; d < D; ++d) e0[d] = tabg[min(d, nsteps - 1) * 4];
    int e_pre = tabg[min(D, nsteps - 1) * 4];
    int ls = D;   // the step whose table entry is e_pre
    f32x4 b4[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
      b4[t] = *reinterpret_cast<const f32x4*>(bias + ft[t] * 16 + g * 4);

    int m[MT], bptr[MT], ooff[MT];
    uint4 rb[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      m[mt] = (pg * MT + mt) * 16 + li;
      const int mc = min(m[mt], M - 1);
      const int pp = div_magic(mc, L.magicQ), qq = mc - pp * Q;
      bptr[mt] = L.in_org + pp * L.in_row + qq * L.in_col;
      ooff[mt] = L.out_org + pp * L.out_row + qq * L.out_col;
      if (has_res) {
        const int roff = L.res_org + pp * L.res_row + qq * L.res_col;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int chunk = min(ft[t] * 2 + (g & 1), (L.res_cs >> 3) - 1);
          rb[mt][t] = *reinterpret_cast<const uint4*>(act + roff + chunk * 16);
        }
      }
    }
    int aptr = a_lane;

    uint4 a[D][NT], b[D][MT];
    auto operands = [&](const int e, uint4* av, uint4* bv) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) bv[mt] = *reinterpret_cast<const uint4*>(act + bptr[mt] + e);
#pragma unroll
      for (int t = 0; t < NT; ++t) av[t] = *reinterpret_cast<const uint4*>(act + aptr + ft[t] * 256);
      aptr += wstep;
    };
#pragma unroll
    for (int d = 0; d < D; ++d)
      if (d < nsteps) operands(e0[d], a[d], b[d]);

    // The accumulator starts from the bias.  The shortcut goes in first: one
    // MFMA step whose filter fragment is one-hot.
    f32x4 acc[MT][NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (has_res && ft[t] * 16 < L.res_cs) {
        const uint4 ia = identity_fragment<BF>(ft[t], L.res_cs, li, g);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][t] = mfma_16x16x32<BF>(ia, rb[mt][t], b4[t]);
      } else {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][t] = b4[t];
      }
    }

    for (int step0 = 0; step0 < nsteps; step0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        if (step0 + d < nsteps) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < NT; ++t)
              acc[mt][t] = mfma_16x16x32<BF>(a[d][t], b[d][mt], acc[mt][t]);
          if (step0 + d + D < nsteps) {
            const int e = e_pre;
            ++ls;
            e_pre = tabg[min(ls, nsteps - 1) * 4];
            operands(e, a[d], b[d]);
          }
        }
      }
    }

    // epilogue: ReLU, one rounding, store
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int k0 = (ft0 + t) * 16 + g * 4;
        if (m[mt] >= M || ft0 + t >= FT || k0 >= ycs) continue;
        float v[4] = {acc[mt][t][0], acc[mt][t][1], acc[mt][t][2], acc[mt][t][3]};
        if (relu) {
          // max(x, 0) on the bit pattern: negative floats are negative integers
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = __int_as_float(max(__float_as_int(v[i]), 0));
        }
        uint2 o;
        o.x = pack2<BF>(v[0], v[1]);
        o.y = pack2<BF>(v[2], v[3]);
        if constexpr (LAST) {
          uint16_t* yp = reinterpret_cast<uint16_t*>(p.y) +
                         ((size_t)n * p.out_pixels + m[mt]) * p.y_cs;
          *reinterpret_cast<uint2*>(yp + k0) = o;
        } else {
          *reinterpret_cast<uint2*>(act + ooff[mt] + k0 * 2) = o;
        }
      }
    }
  }
}

template <bool BF, int MT, int NT>
__device__ __forceinline__ void conv_layer(const ResLayer& L, const ResParams& p, char* act,
                                           int n, int lane, int wave) {
  if (L.flags & kResLast) conv_items<BF, MT, NT, true>(L, p, act, n, lane, wave);
  else conv_items<BF, MT, NT, false>(L, p, act, n, lane, wave);
}

// Global mean over the M interior pixels of the input, per channel, in fp32:
// L.MT partial sums over interleaved pixels, then their sum in order.
template <bool BF>
__device__ __forceinline__ void mean_layer(const ResLayer& L, const ResParams& p, char* lds,
                                           char* act, int n, int tid) {
  float* part = reinterpret_cast<float*>(lds);   // parts x cs_out floats of scratch
  const int cs = L.cs_out, M = L.M, Q = L.Q, parts = L.MT;
  if (tid < parts * cs) {
    const int c = tid % cs, k = tid / cs;
    float acc = 0.f;
    for (int i = k; i < M; i += parts) {
      const int pp = div_magic(i, L.magicQ), qq = i - pp * Q;
      acc += to_float<BF>(*reinterpret_cast<const uint16_t*>(act + L.in_org + pp * L.in_row +
                                                             qq * L.in_col + c * 2));
    }
    part[k * cs + c] = acc;
  }
  __syncthreads();
  if (tid < cs) {
    float acc = 0.f;
    for (int k = 0; k < parts; ++k) acc += part[k * cs + tid];
    const uint16_t o = from_float<BF>(acc / (float)M);
    if (L.flags & kResLast) reinterpret_cast<uint16_t*>(p.y)[(size_t)n * p.y_cs + tid] = o;
    else *reinterpret_cast<uint16_t*>(act + L.out_org + tid * 2) = o;
  }
}

// The layer table is read through the constant address space so that every
// descriptor load is a scalar load (a uniform load from plain global memory
// after the kernel's first store becomes a vector load whose wait would also
// drain the parameter staging in flight).
typedef const uint32_t __attribute__((address_space(4)))* ConstWords;
typedef const void __attribute__((address_space(1)))* GlobalPtr;
typedef void __attribute__((address_space(3)))* LdsPtr;

// The first eight dwords of a ResLayer: all that staging needs.
struct StageHead {
  const void* packed;
  const void* table;
  int32_t blob_units, tab_units, w_off, tab_off;
};
static_assert(sizeof(StageHead) == 32, "StageHead mirrors the head of ResLayer");

template <class T>
__device__ __forceinline__ T load_words(ConstWords w) {
  constexpr int kWords = sizeof(T) / 4;
  struct Raw { uint32_t u[kWords]; } raw;
#pragma unroll
  for (int i = 0; i < kWords; ++i) raw.u[i] = w[i];
  return __builtin_bit_cast(T, raw);
}

// A layer's parameter blob and tap table go from global memory straight into
// LDS (16 bytes per lane, lane i of a wave to the i-th 16-byte slot after the
// wave's base), issued before the current layer is computed and awaited after
// it: no register is held and no global-memory latency sits on the layer chain.
__device__ __forceinline__ void stage_params(const StageHead& H, char* act, int lane, int wave) {
  const char* src = reinterpret_cast<const char*>(H.packed);
  for (int u = wave * 64; u < H.blob_units; u += kResThreads) {
    if (u + lane < H.blob_units)
      __builtin_amdgcn_global_load_lds((GlobalPtr)(src + (size_t)(u + lane) * 16),
                                       (LdsPtr)(act + H.w_off + u * 16), 16, 0, 0);
  }
  // the table (at most 64 slots) goes through the last wave, which has the
  // smallest share of the blob
  if (wave == kWaves - 1 && lane < H.tab_units)
    __builtin_amdgcn_global_load_lds(
        (GlobalPtr)(reinterpret_cast<const char*>(H.table) + lane * 16), (LdsPtr)(act + H.tab_off),
        16, 0, 0);
}

__device__ __forceinline__ void staging_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <bool BF>
__global__ __launch_bounds__(kResThreads) void resident_kernel(const ResParams p) {
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  char* act = lds + kResScratchBytes;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = blockIdx.x;
  ConstWords table = (ConstWords)(uintptr_t)p.layers;
  constexpr int kLayerWords = sizeof(ResLayer) / 4;

  {
    const StageHead H = load_words<StageHead>(table);
    stage_params(H, act, lane, wave);
    // stage the image into the interior of its LDS tensor, zero its halo
    const int cpp = p.in_cs >> 3;
    const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(p.x) +
                                                      (size_t)n * p.in_H * p.in_W * p.in_cs);
    const int total = p.in_H * p.in_W * cpp;
    for (int i = tid; i < total; i += kResThreads) {
      const int pix = i / cpp, ch = i - pix * cpp;
      const int row = pix / p.in_W, col = pix - row * p.in_W;
      *reinterpret_cast<uint4*>(act + p.in_org + (row * p.in_Wh + col) * p.in_ps2 + ch * 16) = src[i];
    }
    if (p.hp > 0 && p.in_H * p.in_W > 1)
      zero_halo(act, p.in_org, p.in_H, p.in_W, p.in_Wh, p.in_ps2, cpp, p.hp, tid);
  }
  ResLayer L = load_words<ResLayer>(table);
  staging_done();
  __syncthreads();

  const int n_layers = p.n_layers;
  for (int l = 0; l < n_layers; ++l) {
    const bool has_next = l + 1 < n_layers;
    if (has_next) {
      const StageHead Hn = load_words<StageHead>(table + (l + 1) * kLayerWords);
      stage_params(Hn, act, lane, wave);
    }

    if (L.flags & kResZeroHalo)
      zero_halo(act, L.hz_org, L.hz_P, L.hz_Q, L.hz_Wh, L.hz_ps2, L.hz_chunks, L.hz_hp, tid);
    if (L.flags & kResMean) {
      mean_layer<BF>(L, p, lds, act, n, tid);
    } else {
      switch (L.MT * 8 + L.NT) {
        case 1 * 8 + 1: conv_layer<BF, 1, 1>(L, p, act, n, lane, wave); break;
        case 1 * 8 + 2: conv_layer<BF, 1, 2>(L, p, act, n, lane, wave); break;
        case 1 * 8 + 3: conv_layer<BF, 1, 3>(L, p, act, n, lane, wave); break;
        case 1 * 8 + 4: conv_layer<BF, 1, 4>(L, p, act, n, lane, wave); break;
        case 2 * 8 + 1: conv_layer<BF, 2, 1>(L, p, act, n, lane, wave); break;
        case 2 * 8 + 2: conv_layer<BF, 2, 2>(L, p, act, n, lane, wave); break;
        case 3 * 8 + 1: conv_layer<BF, 3, 1>(L, p, act, n, lane, wave); break;
        default: conv_layer<BF, 4, 1>(L, p, act, n, lane, wave); break;
      }
    }
    if (has_next) L = load_words<ResLayer>(table + (l + 1) * kLayerWords);   // in flight across the barrier
    staging_done();
    __syncthreads();   // this layer's output and the next layer's parameters are visible
  }
}

std::once_flag g_attr_once;
hipError_t g_attr_status = hipSuccess;

}  // namespace

fupr_status launch_resident(const ResParams& p, int N, fupr_dtype dt, void* stream) {
  std::call_once(g_attr_once, [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&resident_kernel<true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)kResLdsLimit);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&resident_kernel<false>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kResLdsLimit);
    g_attr_status = e;
  });
  if (g_attr_status != hipSuccess) return FUPR_ERR_LAUNCH;
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  if (dt == FUPR_BF16)
    hipLaunchKernelGGL(resident_kernel<true>, dim3(N), dim3(kResThreads), p.lds_bytes, hs, p);
  else
    hipLaunchKernelGGL(resident_kernel<false>, dim3(N), dim3(kResThreads), p.lds_bytes, hs, p);
  return launch_status("resident_kernel");
}

}  // namespace fupr
