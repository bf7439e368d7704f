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

// Pixel addressing of a wave's first work item, kept from one layer to the next:
// consecutive layers of one resolution give a wave the same pixels at the same
// strides, so the divisions and multiplications behind these offsets are done
// once per resolution rather than once per layer.
struct PixelCache {
  int rin[4];    // byte offset of the pixel's window from the window of pixel 0, per pixel tile
};

typedef short short2_t __attribute__((ext_vector_type(2)));

// max(x, floor) on two packed 16-bit floats, as signed 16-bit integers: with
// floor = 0 this is ReLU (negative floats are negative integers), with floor =
// the most negative integer it is the identity.
__device__ __forceinline__ uint32_t clamp_below(uint32_t v, uint32_t floor2) {
  const short2_t a = __builtin_bit_cast(short2_t, v), f = __builtin_bit_cast(short2_t, floor2);
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, f));
}

// All work items of one conv layer that fall to this wave.  LAST: the layer
// writes the network output to global memory instead of LDS.
//
// Every activation tensor in LDS carries a ring of zero pixels as wide as the
// largest padding of any convolution, so a tap never needs a bounds check: the
// K loop is MT + 1 address additions, MT + NT LDS reads and MT * NT MFMAs per
// step, plus one table read per step issued a whole group of steps ahead.  D
// steps of operands are kept in flight (ring of register buffers, loop
// unrolled by D).
template <bool BF, int MT, int NT, bool LAST>
__device__ __forceinline__ void conv_items(const ResLayer& L, const ResParams& p, char* act,
                                           int n, int lane, int wave, PixelCache& pc) {
  constexpr int D = (MT + NT <= 3) ? 4 : (MT + NT == 4 ? 3 : 2);
  const int li = lane & 15, g = lane >> 4;
  const int nsteps = L.nsteps, FT = L.FT, M = L.M, Q = L.Q;
  const bool has_res = L.res_org >= 0;
  const bool full_pixels = (L.flags & kResFullPixels) != 0;     // no pixel tile is ragged
  const bool full_filters = (L.flags & kResFullFilters) != 0;   // no filter tile is missing or partly stored
  const bool reuse = (L.flags & kResReuse) != 0;                // pc holds this layer's first item
  const uint32_t floor2 = (L.flags & kResRelu) ? 0u : 0x80008000u;
  const int ycs = LAST ? p.y_cs : L.cs_out;
  const int wstep = L.wstep;
  const int a_lane = L.wts_off + g * (wstep >> 2) + li * 16;
  const float* bias = reinterpret_cast<const float*>(act + L.w_off);
  const int tab_lane = L.tab_off + g * 4;
  const int n_items = L.n_items, n_fgroups = L.n_fgroups;

  for (int item = wave; item < n_items; item += kWaves) {
    const int pg = div_magic(item, L.magicF);
    const int ft0 = (item - pg * n_fgroups) * NT;
    // filter tiles past the last one repeat it (computed, not stored)
    int ft[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) ft[t] = min(ft0 + t, FT - 1);

    // Table entries of the first two groups of steps and the bias are requested
    // first: their latency passes while the addresses are worked out.  (The
    // table is padded by 2 * D steps, so no index needs clamping.)
    int e0[D], e_cur[D];   // entries of steps 0 .. D-1 and D .. 2D-1
#pragma unroll
    for (int d = 0; d < D; ++d) e0[d] = *reinterpret_cast<const int*>(act + tab_lane + d * 16);
#pragma unroll
    for (int d = 0; d < D; ++d)
      e_cur[d] = *reinterpret_cast<const int*>(act + tab_lane + (D + d) * 16);
    int tptr = tab_lane + 2 * D * 16;
    f32x4 b4[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
      b4[t] = *reinterpret_cast<const f32x4*>(bias + ft[t] * 16 + g * 4);

    int m[MT], rin[MT], rout[MT];
    if (reuse && item == wave) {
      // same pixels, same strides as in the previous layer; output strides = input strides
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        m[mt] = 0;   // not looked at: no pixel tile is ragged
        rin[mt] = pc.rin[mt];
        rout[mt] = rin[mt] + g * 8;
      }
    } else {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        m[mt] = (pg * MT + mt) * 16 + li;
        const int mc = min(m[mt], M - 1);
        const int pp = div_magic(mc, L.magicQ), qq = mc - pp * Q;
        rin[mt] = pp * L.in_row + qq * L.in_col;
        rout[mt] = pp * L.out_row + qq * L.out_col + g * 8;
        pc.rin[mt] = rin[mt];
      }
    }

    // shortcut operands: 16 bytes of the shortcut pixel per lane
    uint4 rb[MT][NT];
    if (has_res) {
      int cres[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t)
        cres[t] = L.res_org + min(ft[t] * 2 + (g & 1), (L.res_cs >> 3) - 1) * 16;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        int rres;
        if (L.flags & kResLikeOut) {
          rres = rout[mt] - g * 8;
        } else {
          const int mc = min(m[mt], M - 1);
          const int pp = div_magic(mc, L.magicQ), qq = mc - pp * Q;
          rres = pp * L.res_row + qq * L.res_col;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t)
          rb[mt][t] = *reinterpret_cast<const uint4*>(act + rres + cres[t]);
      }
    }

    int aptr = a_lane + ft0 * 256;
    uint4 a[D][NT], b[D][MT];
    auto operands = [&](const int e, uint4* av, uint4* bv) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        bv[mt] = *reinterpret_cast<const uint4*>(act + rin[mt] + e);   // e includes the origin
#pragma unroll
      for (int t = 0; t < NT; ++t)
        av[t] = *reinterpret_cast<const uint4*>(act + aptr + (ft[t] - ft0) * 256);
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

    // scheduling hint: one LDS read and one address addition in the shadow of
    // each of the next n MFMAs (a wave alone on its SIMD otherwise issues the
    // MFMAs back to back and only then the reads)
    auto interleave = [](int n) {
#pragma unroll
      for (int i = 0; i < n; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
        __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);   // vector ALU
      }
    };
    auto mfmas = [&](const uint4* av, const uint4* bv) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[mt][t] = mfma_16x16x32<BF>(av[t], bv[mt], acc[mt][t]);
    };
    // The table entries a step needs are read a whole group of D steps ahead
    // of it.  Main part: groups whose D steps and D refills all exist, no
    // condition inside; then at most 2D - 1 steps with conditions.
    int step0 = 0;
    for (; step0 + 2 * D <= nsteps; step0 += D) {
      int e_nxt[D];
#pragma unroll
      for (int d = 0; d < D; ++d) e_nxt[d] = *reinterpret_cast<const int*>(act + tptr + d * 16);
      tptr += D * 16;
#pragma unroll
      for (int d = 0; d < D; ++d) {
        mfmas(a[d], b[d]);
        operands(e_cur[d], a[d], b[d]);
      }
      interleave(D * MT * NT);
#pragma unroll
      for (int d = 0; d < D; ++d) e_cur[d] = e_nxt[d];
    }
    for (; step0 < nsteps; step0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        if (step0 + d < nsteps) {
          mfmas(a[d], b[d]);
          if (step0 + d + D < nsteps) operands(e_cur[d], a[d], b[d]);
        }
      }
    }

    // epilogue: one rounding, ReLU on the rounded pair, store
    if (!LAST && MT % 2 == 0 && full_pixels && full_filters) {
      // Two pixel tiles at a time.  A lane holds 4 channels (8 bytes) of one
      // pixel of each tile; lanes 16 apart hold the next 4 channels of the same
      // pixel.  Swapping odd 16-lane rows of the first tile's registers with
      // even rows of the second's gives every lane 8 consecutive channels of
      // ONE pixel (even rows: first tile, odd rows: second tile): half as many
      // LDS stores, each 16 bytes.
#pragma unroll
      for (int mt = 0; mt < MT; mt += 2) {
        const int wsel = ((g & 1) ? rout[mt + 1] : rout[mt]) - g * 8 + (g >> 1) * 16;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const uint32_t p0 = clamp_below(pack2<BF>(acc[mt][t][0], acc[mt][t][1]), floor2);
          const uint32_t p1 = clamp_below(pack2<BF>(acc[mt][t][2], acc[mt][t][3]), floor2);
          const uint32_t q0 = clamp_below(pack2<BF>(acc[mt + 1][t][0], acc[mt + 1][t][1]), floor2);
          const uint32_t q1 = clamp_below(pack2<BF>(acc[mt + 1][t][2], acc[mt + 1][t][3]), floor2);
          const auto r0 = __builtin_amdgcn_permlane16_swap(p0, q0, false, false);
          const auto r1 = __builtin_amdgcn_permlane16_swap(p1, q1, false, false);
          *reinterpret_cast<uint4*>(act + wsel + (L.out_org + (ft0 + t) * 32)) =
              uint4{r0[0], r1[0], r0[1], r1[1]};
        }
      }
      continue;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        uint2 o;
        o.x = clamp_below(pack2<BF>(acc[mt][t][0], acc[mt][t][1]), floor2);
        o.y = clamp_below(pack2<BF>(acc[mt][t][2], acc[mt][t][3]), floor2);
        const int k0 = (ft0 + t) * 16 + g * 4;
        if (!full_pixels && m[mt] >= M) continue;
        if (!full_filters && (ft0 + t >= FT || k0 >= ycs)) continue;
        if constexpr (LAST) {
          uint16_t* yp = reinterpret_cast<uint16_t*>(p.y) +
                         ((size_t)n * p.out_pixels + m[mt]) * p.y_cs;
          *reinterpret_cast<uint2*>(yp + k0) = o;
        } else {
          *reinterpret_cast<uint2*>(act + rout[mt] + (L.out_org + (ft0 + t) * 32)) = o;
        }
      }
    }
  }
}

template <bool BF, int MT, int NT>
__device__ __forceinline__ void conv_layer(const ResLayer& L, const ResParams& p, char* act,
                                           int n, int lane, int wave, PixelCache& pc) {
  if (L.flags & kResLast) conv_items<BF, MT, NT, true>(L, p, act, n, lane, wave, pc);
  else conv_items<BF, MT, NT, false>(L, p, act, n, lane, wave, pc);
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

// One wave-wide global -> LDS load: lane i moves 16 bytes from its own global
// address to the i-th 16-byte slot after lds_base (M0 holds the base).  Written
// as inline assembly so that the compiler does not take it for an LDS store
// that later LDS reads might alias (it would wait for the whole transfer before
// the current layer's first LDS access); the kernel orders it by hand: issued
// after the barrier that retires the destination's previous contents, awaited
// (vmcnt) before the barrier that publishes it.
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

__device__ __forceinline__ uint32_t lds_address(const char* p) {
  return (uint32_t)(uintptr_t)(LdsPtr)p;
}

// A layer's parameter blob and tap table go from global memory straight into
// LDS, issued before the current layer is computed and awaited after it: no
// register is held and no global-memory latency sits on the layer chain.  The
// waves that have no work item in the current layer (busy = number that do) do
// the staging; when every wave is busy all share it.
__device__ __forceinline__ void stage_params(const StageHead& H, int busy, char* act, int lane,
                                             int wave) {
  const int stagers = busy < kWaves ? kWaves - busy : kWaves;
  const int me = busy < kWaves ? wave - busy : wave;
  if (me < 0) return;
  const char* src = reinterpret_cast<const char*>(H.packed);
  const uint32_t dst = lds_address(act + H.w_off);
  const uint32_t lane_offset = lane * 16;
  for (int u = me * 64; u < H.blob_units; u += stagers * 64) {
    if (u + lane < H.blob_units) load_to_lds(src + (size_t)u * 16, lane_offset, dst + u * 16);
  }
  // the table (at most 64 slots) goes through the last wave, which has the
  // smallest share of the blob
  if (wave == kWaves - 1 && lane < H.tab_units)
    load_to_lds(H.table, lane_offset, lds_address(act + H.tab_off));
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
    stage_params(load_words<StageHead>(table), kWaves, act, lane, wave);
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
  PixelCache pc;
  for (int l = 0; l < n_layers; ++l) {
    const bool has_next = l + 1 < n_layers;
    if (has_next) {
      const StageHead Hn = {L.next_packed, L.next_table, L.next_blob_units,
                            L.next_tab_units, L.next_w_off, L.next_tab_off};
      stage_params(Hn, (L.flags & kResMean) ? kWaves : L.n_items, act, lane, wave);
    }

    if (L.flags & kResZeroHalo)
      zero_halo(act, L.hz_org, L.hz_P, L.hz_Q, L.hz_Wh, L.hz_ps2, L.hz_chunks, L.hz_hp, tid);
    if (L.flags & kResMean) {
      mean_layer<BF>(L, p, lds, act, n, tid);
    } else {
      switch (L.MT * 8 + L.NT) {
        case 1 * 8 + 1: conv_layer<BF, 1, 1>(L, p, act, n, lane, wave, pc); break;
        case 1 * 8 + 2: conv_layer<BF, 1, 2>(L, p, act, n, lane, wave, pc); break;
        case 2 * 8 + 1: conv_layer<BF, 2, 1>(L, p, act, n, lane, wave, pc); break;
        case 2 * 8 + 2: conv_layer<BF, 2, 2>(L, p, act, n, lane, wave, pc); break;
        default: conv_layer<BF, 4, 1>(L, p, act, n, lane, wave, pc); break;
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
