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
// Per layer: the next layer's parameter blob is fetched from global memory into
// registers BEFORE the current layer is computed and written to LDS after it,
// so no global-memory latency sits on the layer chain; both MFMA operands of
// the current layer (filters = A, pixels = B) come from LDS.  A work item is
// MT pixel tiles x NT filter tiles of 16 x 16, so every LDS fragment feeds
// several MFMAs.
//
// Arithmetic is the same as the per-layer kernel's, step for step: the same chunk
// order along (r, s, c), the same MFMA 16x16x32 accumulation, the same
// epilogue (bias, shortcut, ReLU, one rounding), so results are bit-identical
// to the per-layer path.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <mutex>

#include "device_utils.h"
#include "fupr.h"
#include "layout.h"

namespace fupr {
namespace {

constexpr int kWaves = kResThreads / 64;

// A wave-uniform value the optimiser knows nothing about.  The layer table
// stores geometry in bytes; arithmetic on values KNOWN to be bytes was turned
// into packed byte dot products that dropped the sign of a subtracted term
// (tap - r*S came out as tap + r*S), so every field is laundered through a
// scalar move before it enters index arithmetic.
__device__ __forceinline__ int opaque(int v) {
  int r;
  asm volatile("s_mov_b32 %0, %1" : "=s"(r) : "s"(v));
  return r;
}

// A layer descriptor unpacked into scalar registers.
struct LayerRegs {
  const void* packed;
  int in_org, out_org, res_org, w_off, blob_units, nchunk;
  int ps_in, ps_out, ps_res, cs_out, res_cs, Kp;
  int Wh_in, Wh_out, P, Q, S, stride, cpt, nsteps, FT, MT, NT, res_Wh, res_ss, flags, out_halo;
};

__device__ __forceinline__ LayerRegs unpack(const ResLayer& L) {
  LayerRegs r;
  r.packed = L.packed;
  const uint32_t off0 = L.off0, off1 = L.off1, sz = L.sz, ps0 = L.ps0, ps1 = L.ps1, ch = L.ch;
  const uint32_t g0 = L.g0, g1 = L.g1, g2 = L.g2, g3 = L.g3;
  r.in_org = opaque(off0 & 0xffff);   r.out_org = opaque(off0 >> 16);
  r.res_org = opaque(off1 & 0xffff);  r.w_off = opaque(off1 >> 16);
  r.blob_units = opaque(sz & 0xffff); r.nchunk = opaque(sz >> 16);
  r.ps_in = opaque(ps0 & 0xffff);     r.ps_out = opaque(ps0 >> 16);
  r.ps_res = opaque(ps1 & 0xffff);    r.cs_out = opaque(ps1 >> 16);
  r.res_cs = opaque(ch & 0xffff);     r.Kp = opaque(ch >> 16);
  r.Wh_in = opaque(g0 & 255);  r.Wh_out = opaque((g0 >> 8) & 255);
  r.P = opaque((g0 >> 16) & 255);  r.Q = opaque(g0 >> 24);
  r.S = opaque(g1 & 255);  r.stride = opaque((g1 >> 8) & 255);
  r.cpt = opaque((g1 >> 16) & 255);  r.nsteps = opaque(g1 >> 24);
  r.FT = opaque(g2 & 255);  r.MT = opaque((g2 >> 8) & 255);
  r.NT = opaque((g2 >> 16) & 255);  r.res_Wh = opaque(g2 >> 24);
  r.res_ss = opaque(g3 & 255);  r.flags = opaque((g3 >> 8) & 255);
  r.out_halo = opaque((g3 >> 16) & 255);
  return r;
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

// All work items of one conv layer that fall to this wave.  LAST: the layer
// writes the network output to global memory instead of LDS.
//
// Every activation tensor in LDS carries a ring of zero pixels as wide as the
// largest padding of any convolution, so a tap never needs a bounds check: the
// K loop is one table read, MT + NT address additions, MT + NT LDS reads and
// MT * NT MFMAs per step.  D steps of operands are kept in flight (ring of
// register buffers, loop unrolled by D), and the table entry of a step is read
// one issue ahead of that step's operand reads.
template <bool BF, int MT, int NT, bool LAST>
__device__ __forceinline__ void conv_items(const LayerRegs& L, const ResParams& p, char* act,
                                           const int* tab, int n, int lane, int wave) {
  constexpr int D = (MT + NT <= 2) ? 4 : (MT + NT <= 4 ? 3 : 2);
  const int li = lane & 15, g = lane >> 4;
  const int Q = L.Q, nsteps = L.nsteps, FT = L.FT, Kp = L.Kp;
  const bool relu = (L.flags & kResRelu) != 0, has_res = L.res_org != 0xffff;
  const int M = L.P * Q;
  const uint32_t magicQ = 0xffffffffu / (uint32_t)Q + 1u;   // floor(m / Q) = mulhi(m, magicQ), m < 2^16
  const int n_ptiles = (M + 15) >> 4;
  const int n_pgroups = (n_ptiles + MT - 1) / MT;
  const int n_fgroups = (FT + NT - 1) / NT;
  const int n_items = n_pgroups * n_fgroups;
  const int ycs = LAST ? p.y_cs : L.cs_out;

  const int in_org = L.in_org * 16, out_org = L.out_org * 16, res_org = L.res_org * 16;
  const int in_row = L.stride * L.Wh_in * L.ps_in * 2, in_col = L.stride * L.ps_in * 2;
  const int out_row = L.Wh_out * L.ps_out * 2, out_col = L.ps_out * 2;
  const int res_row = L.res_ss * L.res_Wh * L.ps_res * 2, res_col = L.res_ss * L.ps_res * 2;
  const int wblob = L.w_off * 16;
  const float* bias = reinterpret_cast<const float*>(act + wblob);
  const int wts = wblob + (Kp * 4 + 255) / 256 * 256;
  const int wstep = 4 * Kp * 16;   // bytes per MFMA step
  const int* tabg = tab + g;

  for (int item = wave; item < n_items; item += kWaves) {
    const int pg = item / n_fgroups;
    const int ft0 = (item - pg * n_fgroups) * NT;
    int m[MT], bptr[MT], ooff[MT], roff[MT];
    bool pv[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      m[mt] = (pg * MT + mt) * 16 + li;
      pv[mt] = m[mt] < M;
      const int mc = min(m[mt], M - 1);
      const int pp = (int)__umulhi((uint32_t)mc, magicQ), qq = mc - pp * Q;
      bptr[mt] = in_org + pp * in_row + qq * in_col;
      ooff[mt] = out_org + pp * out_row + qq * out_col;
      roff[mt] = res_org + pp * res_row + qq * res_col;
    }
    int aptr[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) aptr[t] = wts + (g * Kp + min(ft0 + t, FT - 1) * 16 + li) * 16;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    uint4 a[D][NT], b[D][MT];
    int ls = 0;   // next step to be issued
    int e_pre;    // its tap-table entry
    auto operands = [&](const int e, uint4* av, uint4* bv) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) bv[mt] = *reinterpret_cast<const uint4*>(act + bptr[mt] + e);
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        av[t] = *reinterpret_cast<const uint4*>(act + aptr[t]);
        aptr[t] += wstep;
      }
      ++ls;
    };

    {
      int e0[D];
#pragma unroll
      for (int d = 0; d < D; ++d) e0[d] = tabg[min(d, nsteps - 1) * 4];
      e_pre = tabg[min(D, nsteps - 1) * 4];
#pragma unroll
      for (int d = 0; d < D; ++d)
        if (d < nsteps) operands(e0[d], a[d], b[d]);
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
          if (ls < nsteps) {
            const int e = e_pre;
            e_pre = tabg[min(ls + 1, nsteps - 1) * 4];
            operands(e, a[d], b[d]);
          }
        }
      }
    }

    // epilogue: bias, shortcut, ReLU, one rounding.  All LDS reads first.
    float4 b4[NT];
    uint2 rv[MT][NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int k0 = (min(ft0 + t, FT - 1)) * 16 + g * 4;
      b4[t] = *reinterpret_cast<const float4*>(bias + k0);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const bool rd = has_res && k0 < L.res_cs;
        rv[mt][t] = rd ? *reinterpret_cast<const uint2*>(act + roff[mt] + k0 * 2) : uint2{0u, 0u};
      }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int k0 = (ft0 + t) * 16 + g * 4;
        if (!pv[mt] || ft0 + t >= FT || k0 >= ycs) continue;
        float v[4] = {acc[mt][t][0] + b4[t].x, acc[mt][t][1] + b4[t].y, acc[mt][t][2] + b4[t].z,
                      acc[mt][t][3] + b4[t].w};
        if (has_res) {
          v[0] += to_float<BF>((uint16_t)(rv[mt][t].x & 0xffffu));
          v[1] += to_float<BF>((uint16_t)(rv[mt][t].x >> 16));
          v[2] += to_float<BF>((uint16_t)(rv[mt][t].y & 0xffffu));
          v[3] += to_float<BF>((uint16_t)(rv[mt][t].y >> 16));
        }
        if (relu) {
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = fmaxf(v[i], 0.f);
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
__device__ __forceinline__ void conv_layer(const LayerRegs& L, const ResParams& p, char* act,
                                           const int* tab, int n, int lane, int wave) {
  if (L.flags & kResLast) conv_items<BF, MT, NT, true>(L, p, act, tab, n, lane, wave);
  else conv_items<BF, MT, NT, false>(L, p, act, tab, n, lane, wave);
}

// A layer's parameter blob: global memory -> registers (issued early) ...
__device__ __forceinline__ void fetch_blob(const void* packed, int units, int tid,
                                           uint4 (&wreg)[kResPrefetch]) {
  const uint4* src = reinterpret_cast<const uint4*>(packed);
#pragma unroll
  for (int k = 0; k < kResPrefetch; ++k) {
    const int idx = tid + k * kResThreads;
    wreg[k] = idx < units ? src[idx] : uint4{0u, 0u, 0u, 0u};
  }
}

// ... and registers -> LDS (after the current layer's compute).
__device__ __forceinline__ void commit_blob(int w_off, int units, int tid, char* act,
                                            const uint4 (&wreg)[kResPrefetch]) {
  uint4* dst = reinterpret_cast<uint4*>(act + w_off * 16);
#pragma unroll
  for (int k = 0; k < kResPrefetch; ++k) {
    const int idx = tid + k * kResThreads;
    if (idx < units) dst[idx] = wreg[k];
  }
}

template <bool BF>
__global__ __launch_bounds__(kResThreads) void resident_kernel(const ResParams p) {
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  int* tables = reinterpret_cast<int*>(lds);   // two tap tables of kResTableEntries
  char* act = lds + 2 * kResTableEntries * sizeof(int);

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n = blockIdx.x;
  const int hp = __builtin_amdgcn_readfirstlane(p.hp);

  // parameters of the layer after the current one travel through these registers
  uint4 wreg[kResPrefetch];
  LayerRegs L = unpack(p.layers[0]);
  fetch_blob(L.packed, L.blob_units, tid, wreg);
  {
    // stage the image into the interior of its LDS tensor, zero its halo
    const int cpp = p.in_cs >> 3;
    const uint4* src = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(p.x) +
                                                      (size_t)n * p.in_H * p.in_W * p.in_cs);
    const int org = p.in_org * 16, ps2 = p.in_ps * 2;
    const int total = p.in_H * p.in_W * cpp;
    for (int i = tid; i < total; i += kResThreads) {
      const int pix = i / cpp, ch = i - pix * cpp;
      const int row = pix / p.in_W, col = pix - row * p.in_W;
      *reinterpret_cast<uint4*>(act + org + (row * p.in_Wh + col) * ps2 + ch * 16) = src[i];
    }
    if (hp > 0 && p.in_H * p.in_W > 1) zero_halo(act, org, p.in_H, p.in_W, p.in_Wh, ps2, cpp, hp, tid);
  }
  commit_blob(L.w_off, L.blob_units, tid, act, wreg);

  const int n_layers = __builtin_amdgcn_readfirstlane(p.n_layers);
  for (int l = 0; l < n_layers; ++l) {
    const bool has_next = l + 1 < n_layers;
    LayerRegs Ln = L;
    if (has_next) {
      Ln = unpack(p.layers[l + 1]);
      fetch_blob(Ln.packed, Ln.blob_units, tid, wreg);
    }

    int* tab = tables + (l & 1) * kResTableEntries;
    if (!(L.flags & kResMean)) {
      const int Wh = L.Wh_in, ps = L.ps_in, cpt = L.cpt, S = L.S;
      const int nentries = L.nsteps * 4, nchunk = L.nchunk;
      for (int j = tid; j < nentries; j += kResThreads) {
        int e = 0;   // padding chunks (zero weights) re-read the first chunk: finite data
        if (j < nchunk) {
          const int tap = j / cpt, c8 = j - tap * cpt;
          const int r = tap / S, s = tap - r * S;
          e = ((r * Wh + s) * ps + c8 * 8) * 2;   // byte offset from the window's first pixel
        }
        tab[j] = e;
      }
    }
    __syncthreads();   // previous layer's output, this layer's parameters and table are visible

    if (L.flags & kResMean) {
      // global mean over the P x Q interior, sequential fp32 sum per channel
      const int Pm = L.P, Qm = L.Q, ps = L.ps_in, Wh = L.Wh_in;
      const uint16_t* in = reinterpret_cast<const uint16_t*>(act + L.in_org * 16);
      for (int c = tid; c < L.cs_out; c += kResThreads) {
        float acc = 0.f;
        for (int i = 0; i < Pm; ++i)
          for (int j = 0; j < Qm; ++j) acc += to_float<BF>(in[(i * Wh + j) * ps + c]);
        const uint16_t o = from_float<BF>(acc / (float)(Pm * Qm));
        if (L.flags & kResLast) reinterpret_cast<uint16_t*>(p.y)[(size_t)n * p.y_cs + c] = o;
        else reinterpret_cast<uint16_t*>(act + L.out_org * 16)[c] = o;
      }
    } else {
      if (L.out_halo > 0 && !(L.flags & kResLast))
        zero_halo(act, L.out_org * 16, L.P, L.Q, L.Wh_out, L.ps_out * 2, L.cs_out >> 3, L.out_halo,
                  tid);
      switch (L.MT * 8 + L.NT) {
        case 1 * 8 + 1: conv_layer<BF, 1, 1>(L, p, act, tab, n, lane, wave); break;
        case 1 * 8 + 2: conv_layer<BF, 1, 2>(L, p, act, tab, n, lane, wave); break;
        case 1 * 8 + 3: conv_layer<BF, 1, 3>(L, p, act, tab, n, lane, wave); break;
        case 1 * 8 + 4: conv_layer<BF, 1, 4>(L, p, act, tab, n, lane, wave); break;
        case 2 * 8 + 1: conv_layer<BF, 2, 1>(L, p, act, tab, n, lane, wave); break;
        case 2 * 8 + 2: conv_layer<BF, 2, 2>(L, p, act, tab, n, lane, wave); break;
        case 3 * 8 + 1: conv_layer<BF, 3, 1>(L, p, act, tab, n, lane, wave); break;
        default: conv_layer<BF, 4, 1>(L, p, act, tab, n, lane, wave); break;
      }
    }
    if (has_next) commit_blob(Ln.w_off, Ln.blob_units, tid, act, wreg);
    L = Ln;
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
