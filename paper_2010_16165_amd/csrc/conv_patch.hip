// 3 x 3 convolution (pad 1, stride 1 or 2) of one layer with the input patch of
// a workgroup staged in LDS (Sec. III, Sec. IV-B-1: operator k x c x 3 x 3; the
// epilogue applies what Sec. VI-B-3 merges and the block's addition and ReLU).
//
// GEMM view as in the other kernels: rows = filters (MFMA operand A), columns =
// output pixels (operand B), reduction over (32-channel stage, tap).
//
//   * The batch is one tall image: image n occupies rows n*Hv + 1 .. n*Hv + H of
//     a virtual input with Hv = H + stride rows per image; the rows between
//     images are zero and serve as the padding of both neighbours.  Output
//     rows are numbered the same way (Pv = P + 1 per image; the extra row is
//     computed and not stored), so a tile is a run of BM consecutive virtual
//     output pixels wherever image boundaries fall, and small images fill
//     their tiles.
//   * A tile's input rows, full width plus a zero column on each side, go
//     global -> LDS 32 channels at a time (two planes of 16 channels, pixel
//     stride 32 bytes: the stride at which 16-byte-per-lane LDS reads run at
//     full rate; for stride 2 even and odd columns are stored apart so that
//     consecutive output pixels still read consecutive slots).  The loads are
//     range-checked buffer loads that write LDS directly: everything outside
//     the image or the tensor arrives as zeros, all lanes always load.
//   * The 9 x 4 weight chunks of the stage for the tile's filters travel the
//     same way; when one filter group covers the layer and all stages' weights
//     fit beside the patch buffers they are loaded once and stay.
//   * Waves are specialised: four loading waves issue the global -> LDS loads
//     of the next unit while the computing waves multiply the current one, so
//     that a computing wave never waits for room in the vector memory queue
//     with its MFMAs behind it.  Units (tile, stage) are double buffered; one
//     barrier per unit joins the two kinds of waves.  The smallest tiles, whose
//     units are shorter than the latency of their loads, keep a ring of up to
//     four buffers and load up to three units ahead.
//   * A workgroup is persistent: it walks a contiguous range of tiles, and the
//     sequence (tile, stage) is one pipeline, so that the first loads of the
//     next tile fly during the last stage and the epilogue of the current one.
//   * Every tap is one MFMA 16x16x32 step whose pixel fragment is an LDS read at
//     (pixel base + row offset + column offset); no range checks in the loop.
//     The accumulators start at zero and the bias joins in the epilogue, so the
//     computing waves touch global memory only there.
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

constexpr int kMaxPatchLoads = 12;          // 16-byte slots of the patch per thread and stage
constexpr uint32_t kOutside = 0x80000000u;  // beyond every tensor this kernel accepts
constexpr size_t kPatchLdsLimit = 160 * 1024;

struct PatchParams {
  const uint16_t* x;
  const uint16_t* w;     // [nchunk_pad][Kp][8]
  const float* bias;
  const uint16_t* res;
  uint16_t* y;
  uint32_t x_bytes, w_bytes, y_bytes, res_bytes;
  int N, H, W, xcs;
  int P, Q, ycs;
  int Hv, Pv, Mv;        // virtual rows per image (input, output); virtual output pixels
  int stride;
  int Kp, cpt, n_stages;
  int rH, rW, rcs, rss, roff;
  int relu;
  const int32_t* keep;   // pruned output filters of a block: filter j adds into channel
  int keep_n, yC;        // keep[j] of y (keep_n ascending entries in 0 .. yC - 1); else nullptr
  int ix_base;           // with keep: LDS byte offset of the computing waves' staging areas
  int PR, Wh, Whh;       // patch rows; slots per patch row (W + 2); even columns per row
  int plane_bytes;       // PR * Wh * 32
  int patch_slots;       // 2 planes * PR * Wh * 2 halves
  int n_loads;           // patch loads per thread and stage
  int tap1, tap2;        // byte offsets of the second and third tap of a row
  int swz;               // 1: the two 16-byte halves of a patch slot are swapped in every second
                         // group of 8 slots (the layout the 32 x 32 tiles read without bank conflicts)
  int w_resident;        // all stages' weights stay in LDS (one filter group only)
  int patch_base;        // LDS byte offset of patch buffer 0
  int buf_stride;        // bytes from one buffer of the ring to the next
  int depth;             // buffers in the ring: units loaded ahead of the one multiplied, plus one
  int fgroups, tiles;
  int tiles_q, tiles_r;  // tiles / grid, tiles % grid
  FastDiv divQ, divWh, divPR, divHv, divPv, divF;   // by Q, Wh, PR, Hv, Pv, fgroups
};

typedef int i32x4 __attribute__((ext_vector_type(4)));

// lane i moves the 16 bytes at offset off of the buffer to the i-th slot after
// lds_base; an offset outside the buffer writes zeros
__device__ __forceinline__ void load_to_lds(const i32x4& rsrc, uint32_t off, uint32_t lds_base) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "buffer_load_dwordx4 %1, %2, 0 offen lds"
      :
      : "s"(lds_base), "v"(off), "s"(rsrc)
      : "memory", "m0");
}

__device__ __forceinline__ i32x4 make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  i32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  r[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
  r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
  r[3] = 0x00020000;
  return r;
}

typedef void __attribute__((address_space(3)))* LdsPtr;
typedef short short2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t clamp_below(uint32_t v, uint32_t floor2) {
  const short2_t a = __builtin_bit_cast(short2_t, v), f = __builtin_bit_cast(short2_t, floor2);
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, f));
}

// s_waitcnt vmcnt(n) for a wave-uniform n known only at run time: wait until at
// most n of this wave's vector-memory loads are outstanding (they complete in
// order).  The counter has 6 bits; a smaller allowance than asked is always safe.
__device__ __forceinline__ void wait_vmcnt(int n) {
#define FUPR_VMCNT(k) case k: asm volatile("s_waitcnt vmcnt(" #k ")" ::: "memory"); break;
  switch (__builtin_amdgcn_readfirstlane(n)) {
    FUPR_VMCNT(0) FUPR_VMCNT(1) FUPR_VMCNT(2) FUPR_VMCNT(3) FUPR_VMCNT(4) FUPR_VMCNT(5) FUPR_VMCNT(6)
    FUPR_VMCNT(7) FUPR_VMCNT(8) FUPR_VMCNT(9) FUPR_VMCNT(10) FUPR_VMCNT(11) FUPR_VMCNT(12)
    FUPR_VMCNT(13) FUPR_VMCNT(14) FUPR_VMCNT(15) FUPR_VMCNT(16) FUPR_VMCNT(17) FUPR_VMCNT(18)
    FUPR_VMCNT(19) FUPR_VMCNT(20) FUPR_VMCNT(21) FUPR_VMCNT(22) FUPR_VMCNT(23) FUPR_VMCNT(24)
    FUPR_VMCNT(25) FUPR_VMCNT(26) FUPR_VMCNT(27) FUPR_VMCNT(28) FUPR_VMCNT(29) FUPR_VMCNT(30)
    FUPR_VMCNT(31) FUPR_VMCNT(32) FUPR_VMCNT(33) FUPR_VMCNT(34) FUPR_VMCNT(35) FUPR_VMCNT(36)
    FUPR_VMCNT(37) FUPR_VMCNT(38) FUPR_VMCNT(39) FUPR_VMCNT(40) FUPR_VMCNT(41) FUPR_VMCNT(42)
    FUPR_VMCNT(43) FUPR_VMCNT(44) FUPR_VMCNT(45) FUPR_VMCNT(46) FUPR_VMCNT(47) FUPR_VMCNT(48)
    default: asm volatile("s_waitcnt vmcnt(48)" ::: "memory"); break;
  }
#undef FUPR_VMCNT
}

constexpr int kLoaderWaves = 4;

// Indexed epilogue: per computing wave, a staging area of 16 pixels x (NT * 16
// slots + 4) floats, a byte table over kIxSpan channels, 64 channel numbers.
constexpr int kIxSpan = 512;
__host__ __device__ constexpr int kIxWaveBytes(int NT) { return 16 * (NT * 64 + 16) + kIxSpan + 256; }

// The loading waves of a workgroup of NWC computing waves whose tile is BM pixels x
// NF filters: they move every unit's weights and input patch global -> LDS, one
// unit (RING: up to p.depth - 1 units) ahead of the computing waves, and meet them
// at one barrier per unit.  lw = number of this wave among the loading waves.
template <int NF, int BM, bool RING>
__device__ __forceinline__ void patch_loader(const PatchParams& p, uint32_t lds_base, int lw, int lane,
                                             int t_begin, int n_units) {
  constexpr int NL = kLoaderWaves * 64;                        // loading threads
  constexpr int kWeightSlots = 36 * NF;                        // 9 taps x 4 chunks x NF filters
  constexpr int kWeightLoads = (kWeightSlots + NL - 1) / NL;
  constexpr int kWeightBytes = kWeightLoads * NL * 16;
  const i32x4 xrsrc = make_rsrc(p.x, p.x_bytes), wrsrc = make_rsrc(p.w, p.w_bytes);
  uint32_t slot_off[kMaxPatchLoads], goff[kMaxPatchLoads];
  int slot_row[kMaxPatchLoads];
  int l_f0 = 0;
  const uint32_t image_row_bytes = (uint32_t)(p.W * p.xcs * 2);
  auto setup_load = [&](int tile) {
    const int strip = div_by(tile, p.divF);
    l_f0 = (tile - strip * p.fgroups) * NF;
    const int gv_lo = div_by(strip * BM, p.divQ);
    const int v0 = gv_lo * p.stride;             // first virtual input row of the patch
    const int n0 = div_by(v0, p.divHv), vrem0 = v0 - n0 * p.Hv;
#pragma unroll
    for (int i = 0; i < kMaxPatchLoads; ++i) {
      if (i < p.n_loads) {
        const int row = slot_row[i] & 0x7fff;
        const int dn = div_by(vrem0 + row, p.divHv);
        const int ihm = vrem0 - dn * p.Hv - 1;   // image row = ihm + row
        const int ih = ihm + row, n = n0 + dn;
        const bool ok = (slot_row[i] & 0x8000) && n < p.N && ih >= 0 && ih < p.H;
        goff[i] = ok ? slot_off[i] + (uint32_t)(n * p.H + ihm) * image_row_bytes : kOutside;
      }
    }
  };
  auto load_weights = [&](int stage, uint32_t wdst) {
#pragma unroll
    for (int i = 0; i < kWeightLoads; ++i) {
      const int sbase = (i * kLoaderWaves + lw) * 64, s = sbase + lane;
      const int row = s / NF, f = s - row * NF;
      const int tap = row >> 2, cc = stage * 4 + (row & 3);
      const bool ok = s < kWeightSlots && cc < p.cpt && l_f0 + f < p.Kp;
      const uint32_t off =
          ok ? (uint32_t)((tap * p.cpt + cc) * p.Kp + l_f0 + f) * 16u : kOutside;
      load_to_lds(wrsrc, off, wdst + sbase * 16);
    }
  };
  auto load_patch = [&](int stage, uint32_t pdst) {
#pragma unroll
    for (int i = 0; i < kMaxPatchLoads; ++i)
      if (i < p.n_loads)
        load_to_lds(xrsrc, goff[i] + (uint32_t)stage * 64u,
                    pdst + ((i * kLoaderWaves + lw) * 64) * 16);
  };

  // the first weights are on their way while the patch slots are worked out
  int l_tile = t_begin, l_stage = 0;
  l_f0 = (l_tile - div_by(l_tile, p.divF) * p.fgroups) * NF;
  if (p.w_resident) {
    for (int st = 0; st < p.n_stages; ++st) load_weights(st, lds_base + st * kWeightBytes);
  } else {
    load_weights(0, lds_base);
  }
  // What a slot of the patch holds does not depend on the tile except for the
  // image row: slot_row = patch row, bit 15 = column inside the image;
  // slot_off = byte offset in x as if patch row 0 were row 0 of image 0.
#pragma unroll
  for (int i = 0; i < kMaxPatchLoads; ++i) {
    slot_off[i] = 0;
    slot_row[i] = 0;
    goff[i] = kOutside;
    if (i < p.n_loads) {
      const int s = (i * kLoaderWaves + lw) * 64 + lane;
      const int t = s >> 1;
      const int t2 = div_by(t, p.divWh), colpos = t - t2 * p.Wh;
      const int plane = div_by(t2, p.divPR), row = t2 - plane * p.PR;
      // which 8 channels the 16 bytes at this position hold: the halves of a slot change
      // places in every second group of 8 slots of a plane when p.swz is set
      const int half = (s & 1) ^ (p.swz & ((row * p.Wh + colpos) >> 3) & 1);
      int col = colpos;
      if (p.stride == 2) {
        const int odd = colpos >= p.Whh ? 1 : 0;
        col = 2 * (colpos - odd * p.Whh) + odd;
      }
      const int iw = col - 1;
      const bool ok = s < p.patch_slots && iw >= 0 && iw < p.W;
      slot_row[i] = row | (ok ? 0x8000 : 0);
      slot_off[i] = (uint32_t)((row * p.W + iw) * p.xcs + plane * 16 + half * 8) * 2u;
    }
  }
  setup_load(l_tile);
  load_patch(0, lds_base + p.patch_base);
  if (++l_stage == p.n_stages) { l_stage = 0; ++l_tile; }
  if constexpr (!RING) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    for (int u = 0; u < n_units; ++u) {
      __syncthreads();   // unit u is in LDS; the computing waves have finished unit u - 1
      if (u + 1 < n_units) {
        if (l_stage == 0) setup_load(l_tile);
        const uint32_t nb = (uint32_t)((u + 1) & 1) * (uint32_t)p.buf_stride;
        if (!p.w_resident) load_weights(l_stage, lds_base + nb);
        load_patch(l_stage, lds_base + p.patch_base + nb);
        if (++l_stage == p.n_stages) { l_stage = 0; ++l_tile; }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
    }
    return;
  }
  // A ring of p.depth buffers: units u + 1 .. u + depth - 1 are on their way while
  // unit u is multiplied.  Loads complete in order, so "unit u + 1 has landed" is
  // "at most the loads of the units after it are outstanding".
  const int per_unit = (p.w_resident ? 0 : kWeightLoads) + p.n_loads;   // loads per thread
  int ring = 1 % p.depth;    // buffer of the next unit to issue
  auto issue = [&]() {
    if (l_stage == 0) setup_load(l_tile);
    const uint32_t nb = (uint32_t)ring * (uint32_t)p.buf_stride;
    if (!p.w_resident) load_weights(l_stage, lds_base + nb);
    load_patch(l_stage, lds_base + p.patch_base + nb);
    if (++l_stage == p.n_stages) { l_stage = 0; ++l_tile; }
    if (++ring == p.depth) ring = 0;
  };
  int issued = 1;
  while (issued < p.depth - 1 && issued < n_units) { issue(); ++issued; }
  wait_vmcnt((issued - 1) * per_unit);
  for (int u = 0; u < n_units; ++u) {
    __syncthreads();   // unit u is in LDS; the computing waves have finished unit u - 1
    if (issued < n_units) { issue(); ++issued; }
    if (u + 1 < n_units) wait_vmcnt((issued - (u + 2)) * per_unit);
  }
  return;
}

// WM x WN computing waves, each owning MT pixel tiles x NT filter tiles of
// 16 x 16, and kLoaderWaves loading waves.  The computing waves issue only LDS
// reads and MFMAs in the main loop (a wave that waits for room in the vector
// memory queue cannot issue its MFMAs); the loading waves move the next unit's
// weights and patch global -> LDS meanwhile.  One barrier per unit joins them.
//
// IX: the indexed epilogue of a block's last convolution whose output filters
// were pruned (p.keep); without it p.keep is not read.
//
// RING: the small tiles, whose units are shorter than the time their loads take
// to arrive, keep a ring of p.depth buffers and load up to depth - 1 units ahead;
// the others use two buffers.
template <bool BF, int WM, int WN, int MT, int NT, bool IX, bool RING>
__global__ __launch_bounds__((WM * WN + kLoaderWaves) * 64) void conv_patch_kernel(
    const PatchParams p) {
  constexpr int NWC = WM * WN;
  constexpr int NL = kLoaderWaves * 64;                        // loading threads
  constexpr int NF = WN * NT * 16;
  constexpr int BM = WM * MT * 16;
  constexpr int kWeightSlots = 36 * NF;                        // 9 taps x 4 chunks x NF filters
  constexpr int kWeightLoads = (kWeightSlots + NL - 1) / NL;
  constexpr int kWeightBytes = kWeightLoads * NL * 16;
  constexpr int kWStep = 4 * NF * 16;                          // bytes of weights per tap
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LdsPtr)lds;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // tiles are dealt in contiguous ranges: tiles_q each, one more for the first tiles_r
  const int wg = blockIdx.x;
  const int t_begin = wg * p.tiles_q + min(wg, p.tiles_r);
  const int t_end = t_begin + p.tiles_q + (wg < p.tiles_r ? 1 : 0);
  const int n_units = (t_end - t_begin) * p.n_stages;
  if (n_units <= 0) return;

  if (wave >= NWC) {
    patch_loader<NF, BM, RING>(p, lds_base, wave - NWC, lane, t_begin, n_units);
    return;
  }

  // ================================ computing waves ================================
  const int li = lane & 15, g = lane >> 4;
  const int wm = wave % WM, wn = wave / WM;
  const __amdgpu_buffer_rsrc_t yrsrc =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.res), 0, p.res_bytes, 0x00020000);
  const int row_bytes = p.Wh * 32;
  int rin[MT];
  uint32_t yoff[MT], roff[MT];   // byte offsets of the pixel in y and in the shortcut tensor
  int c_f0 = 0;
  f32x4 acc[MT][NT], bias4[NT];
  // Epilogue accesses are 16 bytes per lane: a pair of filter tiles (t, t + 1)
  // is exchanged between 16-lane rows, after which lane (pixel, g) holds channels
  // (g >> 1) * 8 .. + 7 of tile t + (g & 1), i.e. a pixel's 64 bytes of the pair
  // come from four lanes of one instruction.  An odd last tile keeps 8 bytes.
  constexpr int NP = NT / 2;
  u32x4 rvw[MT][NP > 0 ? NP : 1];   // shortcut values, fetched during the last stage
  u32x2 rvo[MT];
  // IX: this wave's filters are slots s0 .. s0 + ns - 1 of the index list; lane l < ns
  // holds the channel of slot s0 + l, k_before / k_after the neighbouring entries (-1: none)
  int ix_ns = 0, ix_chan = 0, ix_before = -1, ix_after = -1;
  auto setup_compute = [&](int tile) {
    const int strip = div_by(tile, p.divF);
    c_f0 = (tile - strip * p.fgroups) * NF;
    const int m0 = strip * BM;
    const int gv_lo = div_by(m0, p.divQ);
    const int q_lo = m0 - gv_lo * p.Q;
    const int n_lo = div_by(gv_lo, p.divPv), p_lo = gv_lo - n_lo * p.Pv;
    const int last = p.Mv - 1 - m0;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int ml = (wm * MT + mt) * 16 + li;
      const int t = q_lo + min(ml, last);
      const int dg = div_by(t, p.divQ), qq = t - dg * p.Q;
      rin[mt] = (dg * p.stride * p.Wh + qq) * 32 + (g >> 1) * p.plane_bytes + (g & 1) * 16;
      const int t2 = p_lo + dg, dn = div_by(t2, p.divPv);
      const int pp = t2 - dn * p.Pv, n = n_lo + dn;
      const bool ok = ml <= last && pp < p.P && n < p.N;   // pp = P: the row between two images
      yoff[mt] = ok ? (uint32_t)(((n * p.P + pp) * p.Q + qq) * p.ycs) * 2u : kOutside;
      roff[mt] = ok ? (uint32_t)(((n * p.rH + pp * p.rss) * p.rW + qq * p.rss) * p.rcs) * 2u
                    : kOutside;
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
  const int k_lane = (wn * NT * 16 + g * 4);
  const int k_pair = wn * NT * 16 + (g & 1) * 16 + (g >> 1) * 8;
  const uint32_t floor2 = p.relu ? 0u : 0x80008000u;

  int c_tile = t_begin, c_stage = 0;
  int ring = 0;   // buffer of the unit being multiplied
  for (int u = 0; u < n_units; ++u) {
    __syncthreads();   // unit u is in LDS
    int buf = u & 1;
    if constexpr (RING) {
      buf = ring;
      if (++ring == p.depth) ring = 0;
    }
    if (c_stage == 0) setup_compute(c_tile);
    const bool last = c_stage == p.n_stages - 1;
    if (!IX && last && p.res) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int pr = 0; pr < NP; ++pr) {
          const int rc = c_f0 + k_pair + pr * 32 - p.roff;
          const uint32_t off = (rc >= 0 && rc < p.rcs) ? roff[mt] + (uint32_t)rc * 2u : kOutside;
          rvw[mt][pr] = __builtin_amdgcn_raw_buffer_load_b128(rrsrc, off, 0, 0);
        }
      if constexpr (NT & 1) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const int rc = c_f0 + k_lane + (NT - 1) * 16 - p.roff;
          const uint32_t off = (rc >= 0 && rc < p.rcs) ? roff[mt] + (uint32_t)rc * 2u : kOutside;
          rvo[mt] = __builtin_amdgcn_raw_buffer_load_b64(rrsrc, off, 0, 0);
        }
      }
    }
    // ---- indexed epilogue, part 1 (see part 2 after the taps) ----
    constexpr int kRow = NT * 64 + 16;          // bytes per pixel row of the staging area
    constexpr int kWholeIt = 3, kNarrowIt = 2;  // rounds per pixel tile fetched ahead of use
    constexpr int kPer = kWholeIt * 4 + kNarrowIt;
    // fetched before the last stage's taps where the registers allow, else after them
    constexpr bool kAhead = IX && MT * NT * 4 + 2 * (MT + NT) * 4 + 44 + MT * kPer <= 256;
    constexpr int kBatch = !IX || kAhead ? MT : (MT * NT > 16 ? 2 : 4);
    char* scr = lds + p.ix_base + wave * kIxWaveBytes(NT);
    uint8_t* inv = reinterpret_cast<uint8_t*>(scr + 16 * kRow);     // kIxSpan bytes
    int* chan = reinterpret_cast<int*>(scr + 16 * kRow + kIxSpan);  // 64 entries
    int a0 = 0, a1 = 0, nch = 0, n_lo = 0, n_hi = 0;
    bool wide = false, lo_shared = false, hi_shared = false;
    u32x4 oldw[IX ? kBatch : 1][kWholeIt];
    uint16_t oldn[IX ? kBatch : 1][kNarrowIt];
    auto whole_off = [&](int mt, int cb) {
      const int a = a0 + cb + g;
      const bool whole =
          wide && cb + g < nch && !((a == a0 && lo_shared) || (a == a1 && hi_shared));
      return whole ? yoff[mt] + (uint32_t)a * 16u : kOutside;
    };
    auto narrow_slot = [&](int q) { return q < n_lo ? q : ix_ns - n_hi + (q - n_lo); };
    auto narrow_off = [&](int mt, int q) {
      const int c = q < n_lo + n_hi ? chan[narrow_slot(q)] : -1;
      return (unsigned)c < (unsigned)p.yC ? yoff[mt] + (uint32_t)c * 2u : kOutside;
    };
    auto fetch_old = [&](int m0) {
#pragma unroll
      for (int dm = 0; dm < kBatch; ++dm) {
        const int mt = min(m0 + dm, MT - 1);
#pragma unroll
        for (int it = 0; it < kWholeIt; ++it)
          oldw[dm][it] = __builtin_amdgcn_raw_buffer_load_b128(
              yrsrc, m0 + dm < MT ? whole_off(mt, it * 4) : kOutside, 0, 0);
#pragma unroll
        for (int it = 0; it < kNarrowIt; ++it)
          oldn[dm][it] = __builtin_amdgcn_raw_buffer_load_b16(
              yrsrc, m0 + dm < MT ? narrow_off(mt, g + it * 4) : kOutside, 0, 0);
      }
    };
    if constexpr (IX) {
      if (c_stage == 0) {
        const int s0 = c_f0 + wn * NT * 16;
        ix_ns = min(NT * 16, p.keep_n - s0);
        ix_chan = p.keep[min(max(s0 + lane, 0), p.keep_n - 1)];
        ix_before = s0 > 0 && ix_ns > 0 ? p.keep[s0 - 1] : -1;
        ix_after = ix_ns > 0 && s0 + ix_ns < p.keep_n ? p.keep[s0 + ix_ns] : -1;
      }
      if (last && ix_ns > 0) {
        // The index list is ascending, so the wave's slots cover the channels
        // c_first .. c_last and own every kept channel in between.  A 16-byte
        // chunk (8 channels) of that range that holds no other wave's channel is
        // read, updated and written whole; only the first and last chunk can hold
        // a neighbour's channel.  This wave's channels in such a chunk (the first
        // n_lo and last n_hi slots), and all of them when the range is wider than
        // the byte table chunk channel -> slot, are updated with 2-byte accesses.
        const int ns = ix_ns;
        const int c_first = __builtin_amdgcn_readfirstlane(ix_chan);
        const int c_last = __builtin_amdgcn_readlane(ix_chan, ns - 1);
        a0 = c_first >> 3;
        a1 = c_last >> 3;
        nch = a1 - a0 + 1;
        wide = c_first >= 0 && nch >= 1 && nch * 8 <= kIxSpan;
        lo_shared = ix_before >= 0 && (ix_before >> 3) == a0;
        hi_shared = ix_after >= 0 && (ix_after >> 3) == a1;
        n_lo = ns;
        n_hi = 0;
        if (wide) {
          const bool mine = lane < ns;
          const int in_lo =
              __builtin_popcountll(__builtin_amdgcn_ballot_w64(mine && (ix_chan >> 3) == a0));
          const int in_hi =
              __builtin_popcountll(__builtin_amdgcn_ballot_w64(mine && (ix_chan >> 3) == a1));
          n_lo = lo_shared ? in_lo : 0;
          n_hi = hi_shared ? in_hi : 0;
          if (a1 == a0 && (lo_shared || hi_shared)) { n_lo = ns; n_hi = 0; }
          *reinterpret_cast<uint2*>(inv + lane * 8) = uint2{0xffffffffu, 0xffffffffu};
        }
        chan[lane] = lane < ns ? ix_chan : -1;
        __builtin_amdgcn_wave_barrier();
        if (wide && lane < ns) {
          const unsigned at = (unsigned)(ix_chan - a0 * 8);
          if (at < (unsigned)kIxSpan) inv[at] = (uint8_t)lane;
        }
        __builtin_amdgcn_wave_barrier();
        if constexpr (kAhead) fetch_old(0);
      }
    }
    const char* wts = lds + (p.w_resident ? c_stage * kWeightBytes : buf * p.buf_stride);
    const char* patch = lds + p.patch_base + buf * p.buf_stride;
    // 9 taps = 9 MFMA steps over these 32 channels; the operands of a step are
    // read while the step before it is multiplied
    uint4 a[2][NT], b[2][MT];
    auto operands = [&](int tap, uint4* av, uint4* bv) {
      const int r = tap / 3, sx = tap - r * 3;
      const int off = r * row_bytes + (sx == 0 ? 0 : (sx == 1 ? p.tap1 : p.tap2));
      // in the order the MFMAs below want them
      av[0] = *reinterpret_cast<const uint4*>(wts + a_lane + tap * kWStep);
      bv[0] = *reinterpret_cast<const uint4*>(patch + rin[0] + off);
#pragma unroll
      for (int t = 1; t < NT; ++t)
        av[t] = *reinterpret_cast<const uint4*>(wts + a_lane + tap * kWStep + t * 256);
#pragma unroll
      for (int mt = 1; mt < MT; ++mt)
        bv[mt] = *reinterpret_cast<const uint4*>(patch + rin[mt] + off);
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
      // keep the taps apart: without this the scheduler sinks the next tap's reads
      // behind this tap's MFMAs and the next tap starts by waiting for them
      // (measured 3 - 8 % slower; the 7 x 4 tile is the exception and stays free)
      if constexpr (MT * NT <= 16) __builtin_amdgcn_sched_barrier(0);
    }
    if (IX && last) {
      if constexpr (IX) {
        // part 2: y holds the shortcut; the sums reach lane (pixel, chunk) through
        // this wave's 16 x slots staging area
        const int ns = ix_ns;
        if (ns > 0) {
          const int n_narrow = n_lo + n_hi;
          auto update_whole = [&](int mt, int cb, const u32x4& oldv) {
            const uint2 which = *reinterpret_cast<const uint2*>(inv + (cb + g) * 8);
            u32x4 out;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              uint32_t halves[2];
#pragma unroll
              for (int h = 0; h < 2; ++h) {
                const int e = 2 * j + h;
                const uint32_t slot = ((e < 4 ? which.x : which.y) >> (8 * (e & 3))) & 0xffu;
                const bool has = slot != 0xffu;
                const float add =
                    *reinterpret_cast<const float*>(scr + li * kRow + (has ? slot : 0u) * 4);
                const uint16_t o = (uint16_t)(oldv[j] >> (16 * h));
                float r = to_float<BF>(o) + add;
                if (p.relu) r = fmaxf(r, 0.f);
                halves[h] = has ? (uint32_t)from_float<BF>(r) : (uint32_t)o;
              }
              out[j] = halves[0] | (halves[1] << 16);
            }
            __builtin_amdgcn_raw_buffer_store_b128(out, yrsrc, whole_off(mt, cb), 0, 0);
          };
          auto update_narrow = [&](int mt, int q, uint16_t o) {
            const int sl = narrow_slot(min(q, max(n_narrow - 1, 0)));
            float r = to_float<BF>(o) + *reinterpret_cast<const float*>(scr + li * kRow + sl * 4);
            if (p.relu) r = fmaxf(r, 0.f);
            __builtin_amdgcn_raw_buffer_store_b16(from_float<BF>(r), yrsrc, narrow_off(mt, q), 0, 0);
          };
#pragma unroll
          for (int m0 = 0; m0 < MT; m0 += kBatch) {
            if constexpr (!kAhead) fetch_old(m0);
#pragma unroll
            for (int dm = 0; dm < kBatch; ++dm) {
              const int mt = m0 + dm;
              if (mt < MT) {
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                  f32x4 v = acc[mt][t];
#pragma unroll
                  for (int i = 0; i < 4; ++i) v[i] += bias4[t][i];
                  *reinterpret_cast<f32x4*>(scr + li * kRow + (t * 16 + g * 4) * 4) = v;
                }
                __builtin_amdgcn_wave_barrier();
                if (wide) {
#pragma unroll
                  for (int it = 0; it < kWholeIt; ++it) update_whole(mt, it * 4, oldw[dm][it]);
                }
#pragma unroll
                for (int it = 0; it < kNarrowIt; ++it)
                  if (g + it * 4 < n_narrow) update_narrow(mt, g + it * 4, oldn[dm][it]);
                // longer ranges
                for (int cb = kWholeIt * 4; wide && cb < nch; cb += 4)
                  update_whole(mt, cb,
                               __builtin_amdgcn_raw_buffer_load_b128(yrsrc, whole_off(mt, cb), 0, 0));
                for (int q = g + kNarrowIt * 4; q < n_narrow; q += 4)
                  update_narrow(mt, q,
                                __builtin_amdgcn_raw_buffer_load_b16(yrsrc, narrow_off(mt, q), 0, 0));
              }
            }
          }
        }
      }
      c_stage = 0;
      ++c_tile;
    } else if (last) {
      // bias, shortcut, ReLU, one rounding
      auto finish = [&](const f32x4& av, const f32x4& bv, uint32_t r0, uint32_t r1) {
        float v[4] = {av[0] + bv[0], av[1] + bv[1], av[2] + bv[2], av[3] + bv[3]};
        if (p.res) {
          v[0] += to_float<BF>((uint16_t)(r0 & 0xffffu));
          v[1] += to_float<BF>((uint16_t)(r0 >> 16));
          v[2] += to_float<BF>((uint16_t)(r1 & 0xffffu));
          v[3] += to_float<BF>((uint16_t)(r1 >> 16));
        }
        u32x2 o;
        o[0] = clamp_below(pack2<BF>(v[0], v[1]), floor2);
        o[1] = clamp_below(pack2<BF>(v[2], v[3]), floor2);
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
            ra0 = s0[0]; ra1 = s1[0];   // tile t
            rb0 = s0[1]; rb1 = s1[1];   // tile t + 1
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
        if constexpr (NT & 1) {
          const int t = NT - 1;
          const u32x2 o = finish(acc[mt][t], bias4[t], rvo[mt][0], rvo[mt][1]);
          const int k0 = c_f0 + k_lane + t * 16;
          const uint32_t off = k0 < p.ycs ? yoff[mt] + (uint32_t)k0 * 2u : kOutside;
          __builtin_amdgcn_raw_buffer_store_b64(o, yrsrc, off, 0, 0);
        }
      }
      c_stage = 0;
      ++c_tile;
    } else {
      ++c_stage;
    }
  }
}

// The same kernel on the 32 x 32 x 16 MFMA (half as many MFMA instructions per flop;
// parity-tested, selected only when forced): WM x WN computing waves, each owning
// MT pixel tiles x NT filter tiles of 32 x 32 (16 accumulator registers each).  LDS
// layout, loading waves and pipeline are those of conv_patch_kernel; what differs
// is how a computing wave's lanes address the operands and the results:
//   * a tap is two MFMA steps of 16 channels (one plane of the patch each); lane
//     (index j = lane % 32, half h = lane / 32) reads chunk 2 * step + h of filter j
//     and the 16 bytes at half h of pixel j's slot in plane `step`;
//   * a finished tile holds, per lane, channels 8 b + 4 h .. + 3 (b = 0 .. 3) of
//     pixel j; the two lanes of a pixel exchange halves (v_permlane32_swap) so that
//     each stores 16 bytes: channels 16 pr + 8 h .. + 7, pr = 0, 1.
// Filters are handled in groups of 32 (the packed blob pads them to 16: the other
// 16 rows of a ragged last group are zeros the loading waves supply).
template <bool BF, int WM, int WN, int MT, int NT, bool RING>
__global__ __launch_bounds__((WM * WN + kLoaderWaves) * 64) void conv_patch32_kernel(
    const PatchParams p) {
  constexpr int NWC = WM * WN;
  constexpr int NL = kLoaderWaves * 64;
  constexpr int NF = WN * NT * 32;
  constexpr int BM = WM * MT * 32;
  constexpr int kWeightSlots = 36 * NF;
  constexpr int kWeightLoads = (kWeightSlots + NL - 1) / NL;
  constexpr int kWeightBytes = kWeightLoads * NL * 16;
  constexpr int kWStep = 4 * NF * 16;                          // bytes of weights per tap
  constexpr int kWHalf = 2 * NF * 16;                          // ... per 16-channel step
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LdsPtr)lds;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wg = blockIdx.x;
  const int t_begin = wg * p.tiles_q + min(wg, p.tiles_r);
  const int t_end = t_begin + p.tiles_q + (wg < p.tiles_r ? 1 : 0);
  const int n_units = (t_end - t_begin) * p.n_stages;
  if (n_units <= 0) return;

  if (wave >= NWC) {
    patch_loader<NF, BM, RING>(p, lds_base, wave - NWC, lane, t_begin, n_units);
    return;
  }

  // ================================ computing waves ================================
  const int j = lane & 31, h = lane >> 5;
  const int wm = wave % WM, wn = wave / WM;
  const __amdgpu_buffer_rsrc_t yrsrc =
      __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rrsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.res), 0, p.res_bytes, 0x00020000);
  const int row_bytes = p.Wh * 32;
  int rin[MT];
  uint32_t yoff[MT], roff[MT];
  int c_f0 = 0;
  f32x16 acc[MT][NT];
  auto setup_compute = [&](int tile) {
    const int strip = div_by(tile, p.divF);
    c_f0 = (tile - strip * p.fgroups) * NF;
    const int m0 = strip * BM;
    const int gv_lo = div_by(m0, p.divQ);
    const int q_lo = m0 - gv_lo * p.Q;
    const int n_lo = div_by(gv_lo, p.divPv), p_lo = gv_lo - n_lo * p.Pv;
    const int last = p.Mv - 1 - m0;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int ml = (wm * MT + mt) * 32 + j;
      const int t = q_lo + min(ml, last);
      const int dg = div_by(t, p.divQ), qq = t - dg * p.Q;
      rin[mt] = (dg * p.stride * p.Wh + qq) * 32;       // the pixel's slot; the half is chosen per tap
      const int t2 = p_lo + dg, dn = div_by(t2, p.divPv);
      const int pp = t2 - dn * p.Pv, n = n_lo + dn;
      const bool ok = ml <= last && pp < p.P && n < p.N;   // pp = P: the row between two images
      yoff[mt] = ok ? (uint32_t)(((n * p.P + pp) * p.Q + qq) * p.ycs) * 2u : kOutside;
      roff[mt] = ok ? (uint32_t)(((n * p.rH + pp * p.rss) * p.rW + qq * p.rss) * p.rcs) * 2u
                    : kOutside;
#pragma unroll
      for (int t32 = 0; t32 < NT; ++t32)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mt][t32][v] = 0.f;
    }
  };
  const int a_lane = h * (NF * 16) + (wn * NT * 32 + j) * 16;
  const int h16 = h * 16;
  const int k_lane = wn * NT * 32 + h * 8;       // first channel of this lane's 16 bytes, pair 0 of tile 0
  const uint32_t floor2 = p.relu ? 0u : 0x80008000u;

  int c_tile = t_begin, c_stage = 0;
  int ring = 0;
  for (int u = 0; u < n_units; ++u) {
    __syncthreads();   // unit u is in LDS
    int buf = u & 1;
    if constexpr (RING) {
      buf = ring;
      if (++ring == p.depth) ring = 0;
    }
    if (c_stage == 0) setup_compute(c_tile);
    const bool last = c_stage == p.n_stages - 1;
    const char* wts = lds + (p.w_resident ? c_stage * kWeightBytes : buf * p.buf_stride);
    const char* patch = lds + p.patch_base + buf * p.buf_stride;
    // 9 taps x 2 steps of 16 channels; the operands of a step are read while the step
    // before it is multiplied
    uint4 a[2][NT], b[2][MT];
    // A slot's two halves are swapped in every second group of 8 slots (bit 8 of the slot's
    // byte offset), so that the 32 lanes that read one half of 32 pixels use every LDS bank
    // equally: half h of the slot at byte offset A is at A ^ (h << 4) ^ ((A >> 4) & 16).
    auto pixel_at = [&](int mt, int off) {
      const int A = rin[mt] + off;
      return A ^ h16 ^ ((A >> 4) & 16);
    };
    auto operands = [&](int step, uint4* av, uint4* bv) {
      const int tap = step >> 1, hs = step & 1;
      const int r = tap / 3, sx = tap - r * 3;
      const int off = r * row_bytes + (sx == 0 ? 0 : (sx == 1 ? p.tap1 : p.tap2));
      const char* plane = patch + hs * p.plane_bytes;
      av[0] = *reinterpret_cast<const uint4*>(wts + a_lane + tap * kWStep + hs * kWHalf);
      bv[0] = *reinterpret_cast<const uint4*>(plane + pixel_at(0, off));
#pragma unroll
      for (int t = 1; t < NT; ++t)
        av[t] = *reinterpret_cast<const uint4*>(wts + a_lane + tap * kWStep + hs * kWHalf + t * 512);
#pragma unroll
      for (int mt = 1; mt < MT; ++mt)
        bv[mt] = *reinterpret_cast<const uint4*>(plane + pixel_at(mt, off));
    };
    operands(0, a[0], b[0]);
#pragma unroll
    for (int step = 0; step < 18; ++step) {
      if (step + 1 < 18) operands(step + 1, a[(step + 1) & 1], b[(step + 1) & 1]);
      // the next step's reads stay in front of this step's MFMAs: left alone, the scheduler
      // sinks every read to just before its use to save registers, and each MFMA then waits
      // out an LDS round trip
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t)
          acc[mt][t] = mfma_32x32x16<BF>(a[step & 1][t], b[step & 1][mt], acc[mt][t]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (!last) {
      ++c_stage;
      continue;
    }
    // ---- epilogue: bias, shortcut, ReLU, one rounding, 16-byte stores ----
    // The shortcut values of the next (filter tile, pixel tile) are fetched while the
    // current one is finished.  (y may be the shortcut's own buffer: a lane then reads
    // exactly the bytes it writes later, and never bytes another element writes.)
    auto load_res = [&](int e, u32x4* rv) {
      const int t = e / MT, mt = e - t * MT;
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        const int rc = c_f0 + k_lane + t * 32 + pr * 16 - p.roff;
        const uint32_t off = (rc >= 0 && rc < p.rcs) ? roff[mt] + (uint32_t)rc * 2u : kOutside;
        rv[pr] = __builtin_amdgcn_raw_buffer_load_b128(rrsrc, off, 0, 0);
      }
    };
    u32x4 rv[2][2];
    if (p.res) load_res(0, rv[0]);
#pragma unroll
    for (int e = 0; e < NT * MT; ++e) {
      const int t = e / MT, mt = e - t * MT;
      if (p.res && e + 1 < NT * MT) load_res(e + 1, rv[(e + 1) & 1]);
      const int kt = c_f0 + (wn * NT + t) * 32;          // first filter of this 32-row tile
      f32x4 bias4[4];
#pragma unroll
      for (int bb = 0; bb < 4; ++bb)
        bias4[bb] = *reinterpret_cast<const f32x4*>(p.bias + min(kt + 8 * bb + 4 * h, p.Kp - 4));
#pragma unroll
      for (int pr = 0; pr < 2; ++pr) {
        // shortcut values into the accumulators' layout: the lanes of a pixel exchange halves
        uint32_t ra[2] = {0u, 0u}, rb[2] = {0u, 0u};
        if (p.res) {
          const u32x4 r4 = rv[e & 1][pr];
          const auto s0 = __builtin_amdgcn_permlane32_swap(r4[0], r4[2], false, false);
          const auto s1 = __builtin_amdgcn_permlane32_swap(r4[1], r4[3], false, false);
          ra[0] = s0[0]; ra[1] = s1[0];   // group 2 pr
          rb[0] = s0[1]; rb[1] = s1[1];   // group 2 pr + 1
        }
        auto finish = [&](int bb, const uint32_t* r) {
          float v[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = acc[mt][t][4 * bb + i] + bias4[bb][i];
          if (p.res) {
            v[0] += to_float<BF>((uint16_t)(r[0] & 0xffffu));
            v[1] += to_float<BF>((uint16_t)(r[0] >> 16));
            v[2] += to_float<BF>((uint16_t)(r[1] & 0xffffu));
            v[3] += to_float<BF>((uint16_t)(r[1] >> 16));
          }
          u32x2 o;
          o[0] = clamp_below(pack2<BF>(v[0], v[1]), floor2);
          o[1] = clamp_below(pack2<BF>(v[2], v[3]), floor2);
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
    }
    c_stage = 0;
    ++c_tile;
  }
}

// Tiles the indexed epilogue is used with.  The two largest leave few registers
// beside their accumulators, fetch from y in small batches and were measured
// slower than the next smaller tiles (27 against 31 us on a 28 x 28, 90 -> 90 of
// 128 layer at batch 64).
constexpr bool indexed_tile(int MT, int NT) { return MT * NT < 21; }

struct PatchTile {
  int WM, WN, MT, NT;    // computing waves along pixels / filters; MFMA tiles per wave
  const char* name;
  bool wide;             // MFMA tiles of 32 x 32 (conv_patch32_kernel), else 16 x 16
};
// MFMA issue clocks per SIMD in the estimates below (short runs of either shape issue close
// to the peak rate: 17 - 19 clocks per 16 x 16 x 32, 34 - 37 per 32 x 32 x 16, measured).
constexpr double kMfmaClocks16 = 16.0, kMfmaClocks32 = 33.0;
// Tiles small enough that a unit's arithmetic is shorter than the latency of its loads.
constexpr bool ring_tile(int NW, int MT, int NT) { return NW * MT * NT <= 16; }
// pixels x filters per workgroup
constexpr PatchTile kTiles[] = {
    {4, 1, 4, 4, "conv3x3p_256x64"}, {4, 1, 4, 3, "conv3x3p_256x48"},
    {4, 1, 4, 2, "conv3x3p_256x32"}, {2, 2, 4, 2, "conv3x3p_128x64"},
    {2, 2, 4, 1, "conv3x3p_128x32"}, {2, 2, 2, 2, "conv3x3p_64x64"},
    {2, 2, 7, 2, "conv3x3p_224x64"}, {2, 2, 7, 1, "conv3x3p_224x32"},
    {4, 1, 7, 4, "conv3x3p_448x64"}, {4, 1, 2, 4, "conv3x3p_128x64w"},
    {4, 1, 7, 2, "conv3x3p_448x32"}, {4, 1, 7, 3, "conv3x3p_448x48"},
    {2, 2, 2, 1, "conv3x3p_64x32"},
    // on the 32 x 32 x 16 MFMA
    {2, 2, 7, 1, "conv3x3q_448x64", true}, {4, 1, 2, 2, "conv3x3q_256x64", true},
    {4, 1, 2, 1, "conv3x3q_256x32", true}, {2, 2, 2, 1, "conv3x3q_128x64", true},
    {2, 2, 1, 1, "conv3x3q_64x64", true},  {4, 1, 1, 2, "conv3x3q_128x64w", true},
    {4, 1, 4, 1, "conv3x3q_512x32", true}, {4, 1, 3, 2, "conv3x3q_384x64", true},
};
// the 32 x 32 tiles whose units are shorter than the latency of their loads
constexpr bool ring_tile32(int NW, int MT, int NT) { return NW * MT * NT <= 8; }
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
// Clocks from issuing a unit's loads to their arrival in LDS (measured on one-image
// layers, whose 16 dependent units of a 64 x 64 tile take 2250 clocks each).
constexpr double kLoadLatency = 2250.0;

int num_compute_units() {
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

struct PatchPlan {
  PatchParams p;
  size_t lds_bytes;
  int grid;
  double cost;
};

// Fills the parameters that depend on the tile; false if the layer does not fit.
bool plan_patch(const Conv16Params& c, int N, const PatchTile& tile, PatchPlan* out) {
  PatchParams p{};
  const int NTH = kLoaderWaves * 64;   // loading threads
  const int NW = tile.WM * tile.WN;
  const int edge = tile.wide ? 32 : 16;
  const int BM = tile.WM * tile.MT * edge, NF = tile.WN * tile.NT * edge;
  if (c.P * c.stride != c.H) return false;
  if (c.res && c.roff % 8 != 0) return false;   // 16-byte shortcut loads
  if (c.keep && (tile.wide || !indexed_tile(tile.MT, tile.NT))) return false;
  p.x = c.x; p.w = c.w; p.bias = c.bias; p.res = c.res; p.y = c.y;
  p.x_bytes = c.x_bytes; p.w_bytes = c.w_bytes;
  p.N = N; p.H = c.H; p.W = c.W; p.xcs = c.xcs;
  p.P = c.P; p.Q = c.Q; p.ycs = c.ycs;
  p.stride = c.stride;
  p.Hv = c.H + c.stride;
  p.Pv = c.P + 1;
  const int64_t Mv = (int64_t)N * p.Pv * c.Q;
  if (Mv >= (int64_t(1) << 30) || (int64_t)N * p.Hv >= (int64_t(1) << 30)) return false;
  const uint64_t y_bytes = (uint64_t)N * c.P * c.Q * c.ycs * 2;
  const uint64_t res_bytes = c.res ? (uint64_t)N * c.rH * c.rW * c.rcs * 2 : 0;
  if ((uint64_t)N * c.H * c.W * c.xcs * 2 >= kOutside || y_bytes >= kOutside ||
      res_bytes >= kOutside)
    return false;
  p.y_bytes = (uint32_t)y_bytes;
  p.res_bytes = (uint32_t)res_bytes;
  p.Mv = (int)Mv;
  p.Kp = c.Kp; p.cpt = c.cpt; p.n_stages = (c.cpt + 3) / 4;
  p.rH = c.rH; p.rW = c.rW; p.rcs = c.rcs; p.rss = c.rss; p.roff = c.roff;
  p.relu = c.relu;
  p.keep = c.keep; p.keep_n = c.keep_n; p.yC = c.yC;
  // virtual output rows a tile can touch
  const int rows_out = BM % c.Q == 0 ? BM / c.Q : (BM - 1 + c.Q - 1) / c.Q + 1;
  p.PR = (rows_out - 1) * c.stride + 3;
  p.Wh = c.W + 2;
  p.Whh = (p.Wh + 1) / 2;
  p.plane_bytes = p.PR * p.Wh * 32;
  p.patch_slots = 2 * p.PR * p.Wh * 2;
  p.n_loads = (p.patch_slots + NTH - 1) / NTH;
  if (p.n_loads > kMaxPatchLoads) return false;
  p.tap1 = c.stride == 1 ? 32 : p.Whh * 32;
  p.tap2 = c.stride == 1 ? 64 : 32;
  const int weight_bytes = (36 * NF + NTH - 1) / NTH * NTH * 16;   // one stage, as loaded
  const int patch_bytes = p.n_loads * NTH * 16;
  p.fgroups = (c.Kp + NF - 1) / NF;
  p.divF = fast_div(p.fgroups);
  // weights of all stages resident when one filter group covers the layer and
  // they fit beside the two patch buffers
  p.swz = tile.wide ? 1 : 0;
  p.w_resident = p.fgroups == 1 &&
                 (size_t)p.n_stages * weight_bytes + 2 * (size_t)patch_bytes <= kPatchLdsLimit;
  const size_t ix_bytes = p.keep ? (size_t)NW * kIxWaveBytes(tile.NT) : 0;
  // Estimated clocks of a unit's arithmetic (see below); a unit shorter than the
  // time its loads take to arrive is worth loading further ahead, LDS permitting.
  const double mfma = tile.wide ? 18.0 * tile.MT * tile.NT * kMfmaClocks32 * NW / 4.0
                                : 9.0 * tile.MT * tile.NT * kMfmaClocks16 * NW / 4.0;
  const double ldsr = (tile.wide ? 18.0 : 9.0) * (tile.MT + tile.NT) * NW * 5.4;
  const bool ring = tile.wide ? ring_tile32(NW, tile.MT, tile.NT) : ring_tile(NW, tile.MT, tile.NT);
  const int want = !ring || mfma + ldsr >= kLoadLatency ? 2 : (mfma + ldsr >= kLoadLatency / 2 ? 3 : 4);
  if (p.w_resident) {
    p.patch_base = p.n_stages * weight_bytes;
    p.buf_stride = patch_bytes;
    const int64_t room = (int64_t)kPatchLdsLimit - (int64_t)ix_bytes - p.patch_base;
    p.depth = (int)std::max<int64_t>(2, std::min<int64_t>(want, room / patch_bytes));
    out->lds_bytes = (size_t)p.patch_base + (size_t)p.depth * (size_t)patch_bytes;
  } else {
    p.patch_base = weight_bytes;
    p.buf_stride = weight_bytes + patch_bytes;
    const int64_t room = (int64_t)kPatchLdsLimit - (int64_t)ix_bytes;
    p.depth = (int)std::max<int64_t>(2, std::min<int64_t>(want, room / p.buf_stride));
    out->lds_bytes = (size_t)p.depth * (size_t)p.buf_stride;
  }
  if (p.keep) {
    p.ix_base = (int)out->lds_bytes;
    out->lds_bytes += ix_bytes;
  }
  p.divQ = fast_div(c.Q);
  p.divWh = fast_div(p.Wh);
  p.divPR = fast_div(p.PR);
  p.divHv = fast_div(p.Hv);
  p.divPv = fast_div(p.Pv);
  if (out->lds_bytes > kPatchLdsLimit) return false;
  const int64_t strips = (Mv + BM - 1) / BM;
  const int64_t tiles = strips * p.fgroups;
  if (tiles >= (int64_t(1) << 30)) return false;
  p.tiles = (int)tiles;
  const int cus = num_compute_units();
  out->grid = (int)std::min<int64_t>(tiles, cus);
  p.tiles_q = p.tiles / out->grid;
  p.tiles_r = p.tiles % out->grid;
  // Estimated clocks.  Measured on gfx950: within a unit the MFMAs and the LDS
  // reads of a computing wave add up rather than overlap (reads issued between
  // MFMAs slow both), a 16-byte-per-lane LDS read costs about 5.4 clocks of the
  // LDS port, the loading waves move about 40 bytes per clock, and the
  // epilogue's 8-byte accesses about 16.
  const double load = (patch_bytes + (p.w_resident ? 0 : weight_bytes)) / 40.0;
  const double unit = std::max({mfma + ldsr, load, kLoadLatency / (p.depth - 1)}) + 150.0;
  const double epi = 500.0 + (double)BM * NF * (c.res ? 4.0 : 2.0) / 16.0;
  const double per_tile = p.n_stages * unit + epi;
  out->cost = 6000.0 + (double)((tiles + out->grid - 1) / out->grid) * per_tile;
  out->p = p;
  return true;
}

template <bool BF, int WM, int WN, int MT, int NT, bool IX>
fupr_status launch_patch_as(const PatchPlan& plan, hipStream_t st) {
  constexpr bool RING = ring_tile(WM * WN, MT, NT);
  static std::once_flag once;
  static hipError_t status = hipSuccess;
  std::call_once(once, [] {
    status = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&conv_patch_kernel<BF, WM, WN, MT, NT, IX, RING>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPatchLdsLimit);
  });
  if (status != hipSuccess) return FUPR_ERR_LAUNCH;
  hipLaunchKernelGGL((conv_patch_kernel<BF, WM, WN, MT, NT, IX, RING>), dim3((unsigned)plan.grid),
                     dim3((WM * WN + kLoaderWaves) * 64), plan.lds_bytes, st, plan.p);
  return launch_status("conv_patch_kernel");
}

template <bool BF, int WM, int WN, int MT, int NT>
fupr_status launch_patch(const PatchPlan& plan, hipStream_t st) {
  if constexpr (indexed_tile(MT, NT)) {
    if (plan.p.keep) return launch_patch_as<BF, WM, WN, MT, NT, true>(plan, st);
  }
  return plan.p.keep ? FUPR_ERR_LIMIT : launch_patch_as<BF, WM, WN, MT, NT, false>(plan, st);
}

template <bool BF, int WM, int WN, int MT, int NT>
fupr_status launch_patch32(const PatchPlan& plan, hipStream_t st) {
  constexpr bool RING = ring_tile32(WM * WN, MT, NT);
  if (plan.p.keep) return FUPR_ERR_LIMIT;
  static std::once_flag once;
  static hipError_t status = hipSuccess;
  std::call_once(once, [] {
    status = hipFuncSetAttribute(
        reinterpret_cast<const void*>(&conv_patch32_kernel<BF, WM, WN, MT, NT, RING>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPatchLdsLimit);
  });
  if (status != hipSuccess) return FUPR_ERR_LAUNCH;
  hipLaunchKernelGGL((conv_patch32_kernel<BF, WM, WN, MT, NT, RING>), dim3((unsigned)plan.grid),
                     dim3((WM * WN + kLoaderWaves) * 64), plan.lds_bytes, st, plan.p);
  return launch_status("conv_patch32_kernel");
}

template <bool BF>
fupr_status dispatch_patch(int tile, const PatchPlan& plan, hipStream_t st) {
  switch (tile) {
    case 13: return launch_patch32<BF, 2, 2, 7, 1>(plan, st);
    case 14: return launch_patch32<BF, 4, 1, 2, 2>(plan, st);
    case 15: return launch_patch32<BF, 4, 1, 2, 1>(plan, st);
    case 16: return launch_patch32<BF, 2, 2, 2, 1>(plan, st);
    case 17: return launch_patch32<BF, 2, 2, 1, 1>(plan, st);
    case 18: return launch_patch32<BF, 4, 1, 1, 2>(plan, st);
    case 19: return launch_patch32<BF, 4, 1, 4, 1>(plan, st);
    case 20: return launch_patch32<BF, 4, 1, 3, 2>(plan, st);
    case 0: return launch_patch<BF, 4, 1, 4, 4>(plan, st);
    case 1: return launch_patch<BF, 4, 1, 4, 3>(plan, st);
    case 2: return launch_patch<BF, 4, 1, 4, 2>(plan, st);
    case 3: return launch_patch<BF, 2, 2, 4, 2>(plan, st);
    case 4: return launch_patch<BF, 2, 2, 4, 1>(plan, st);
    case 5: return launch_patch<BF, 2, 2, 2, 2>(plan, st);
    case 6: return launch_patch<BF, 2, 2, 7, 2>(plan, st);
    case 7: return launch_patch<BF, 2, 2, 7, 1>(plan, st);
    case 8: return launch_patch<BF, 4, 1, 7, 4>(plan, st);
    case 9: return launch_patch<BF, 4, 1, 2, 4>(plan, st);
    case 10: return launch_patch<BF, 4, 1, 7, 2>(plan, st);
    case 11: return launch_patch<BF, 4, 1, 7, 3>(plan, st);
    case 12: return launch_patch<BF, 2, 2, 2, 1>(plan, st);
    default: return FUPR_ERR_LIMIT;
  }
}

bool patch_disabled() {
  return tuning_off("conv_patch");
}

// The tile with the least estimated time; the tuning switch patch_tile=<index> forces one
// (tuning aid).  -1: none fits.
int pick_patch(const Conv16Params& c, int N, PatchPlan* best) {
  const int forced = tuning_int("patch_tile", -1);
  int which = -1;
  for (int i = 0; i < kNumTiles; ++i) {
    PatchPlan plan;
    if (!plan_patch(c, N, kTiles[i], &plan)) continue;
    if (i == forced) {
      *best = plan;
      return i;
    }
    // The 32 x 32 tiles run when forced only: on every 3 x 3 layer of the ResNet-18 / ResNet-50
    // workloads the best of them was measured equal to or slower than the best 16 x 16 tile
    // (47.9 against 54.0 us, 15.9 against 18.3 us, 22.4 against 22.4 us, ...): these layers are
    // bound by what the loading waves can bring into LDS per unit, not by MFMA issue.
    if (kTiles[i].wide) continue;
    // equal estimates at stride 2 go to the later tile: there 64 x 64 beats 128 x 32 and the
    // 4 x 1 arrangement of 128 x 64 beats the 2 x 2 one (measured on the stride-2 layers of the
    // ResNet-18 / ResNet-50 workloads: 15.4 against 21.0 us, 14.4 against 16.0 us)
    if (which < 0 || plan.cost < best->cost || (c.stride == 2 && plan.cost <= best->cost)) {
      *best = plan;
      which = i;
    }
  }
  return which;
}

}  // namespace

bool conv_patch_applies(const Conv16Params& c, int N) {
  if (patch_disabled()) return false;
  if (c.S != 3 || c.nchunk != 9 * c.cpt || c.pad != 1 || (c.stride != 1 && c.stride != 2))
    return false;
  if (c.cpt < 2) return false;   // fewer than 16 channels: nothing to reuse
  PatchPlan plan;
  const int t = pick_patch(c, N, &plan);
  if (t < 0) return false;
  // Stride 2 needs four input pixels per output pixel in LDS, once per filter group, which
  // leaves small tiles.  Where those come in rounds, the general kernel, which reads pixel
  // fragments straight from global memory, was measured equal or faster (128 -> 180 channels at
  // 28 x 28, batch 64: 19.0 against 24.8 us; 256 -> 359 at 14 x 14, batch 256: 50 against 59 us;
  // at most 4 % slower where the filter count is a multiple of 64).  A single round of tiles
  // stays here (256 -> 359 at 14 x 14, batch 64: 22 against 31 us), and so does a layer of one
  // image, a chain of dependent units that this kernel loads further ahead.
  if (c.stride == 2 && plan.p.tiles > plan.grid) return false;
  return true;
}

const char* conv_patch_name(const Conv16Params& c, int N) {
  PatchPlan plan;
  const int t = pick_patch(c, N, &plan);
  return t < 0 ? "conv3x3p" : kTiles[t].name;
}

fupr_status launch_conv_patch(const Conv16Params& c, int N, bool bf16, void* stream) {
  PatchPlan plan;
  const int t = pick_patch(c, N, &plan);
  if (t < 0) return FUPR_ERR_LIMIT;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  return bf16 ? dispatch_patch<true>(t, plan, st) : dispatch_patch<false>(t, plan, st);
}

}  // namespace fupr
