// Whole-network executor: validates an operator list, plans which intermediate
// tensors share workspace memory, and enqueues one kernel per operator on the
// caller's stream (Table II networks after fusion and filter removal).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <array>
#include <cstdio>
#include <cstdlib>
#include <mutex>
#include <new>
#include <vector>

#include "fupr.h"
#include "layout.h"
#include "stem_pool.h"
#include "tuning.h"

using namespace fupr;

namespace {

struct TensorInfo {
  int C, H, W, cs;   // per image
  int buffer;        // workspace buffer id; -1 = network input, -2 = network output
  int last_use;      // index of the last operator reading it
};

}  // namespace

constexpr int kMaxSplit = 4;

struct fupr_model {
  fupr_dtype dt;
  std::vector<fupr_op_desc> ops;
  std::vector<TensorInfo> tensors;        // n_ops + 1
  std::vector<size_t> buffer_elems;       // per image, per workspace buffer
  int schedule = FUPR_SCHEDULE_AUTO;
  bool resident_ok = false;               // the whole network fits one LDS-resident kernel
  ResParams resident{};                   // x, y, y_cs filled per call
  std::vector<ResLayer> res_layers;       // host copy of the layer table
  std::vector<int32_t> res_tables;        // tap tables of all layers, back to back
  std::vector<size_t> res_table_at;       // first entry of each layer's table
  const void* res_dev = nullptr;          // the caller's device copy of the table (fupr_model_set_table)
  // Per-operator schedule: the batch runs as sub-batches on streams the caller
  // lends (fupr_model_set_side_streams) that fork from and join the caller's
  // stream, so that one sub-batch's launch gaps, prologues and tails are filled
  // by the other's work.
  int n_side = 0;
  hipStream_t side_stream[kMaxSplit - 1] = {};
  hipEvent_t fork_event = nullptr, join_event[kMaxSplit - 1] = {};
  std::mutex side_mutex;                  // one forked enqueue at a time: the events are shared
};

struct fupr_graph {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};

namespace {

// Shape of one work item of the LDS-resident kernel for a conv layer: MT pixel
// tiles x NT filter tiles.  Picks the shape with the smallest estimated layer
// time from three measured rates: the compute unit's LDS port (about 5.6 clocks
// per 1 KB fragment read, 16 per 8-byte-per-lane store), MFMA 16x16x32 issue on
// the busiest of the four SIMDs (16 clocks, 24 when a wave has a single
// accumulator and every MFMA waits for the one before), and vector
// instructions beside them (about 2.7 clocks each).  Items go round robin
// over 16 waves, hence over the 4 SIMDs.
// The tuning switch res_item="M/FT/nsteps:MTxNT,..." overrides the choice per
// layer class (an aid for sweeps).
void resident_item_shape(int M, int FT, int nsteps, bool has_res, int* MT_out, int* NT_out) {
  static const int shapes[5][2] = {{4, 1}, {2, 2}, {2, 1}, {1, 2}, {1, 1}};
  char env[128];
  if (tuning_text("res_item", env, sizeof(env))) {
    const char* c = env;
    while (*c) {
      int em = 0, ef = 0, es = 0, mt = 0, nt = 0, used = 0;
      if (std::sscanf(c, "%d/%d/%d:%dx%d%n", &em, &ef, &es, &mt, &nt, &used) == 5) {
        if (em == M && ef == FT && es == nsteps)
          for (const auto& sh : shapes)
            if (sh[0] == mt && sh[1] == nt) { *MT_out = mt; *NT_out = nt; return; }
        c += used;
      }
      while (*c && *c != ',') ++c;
      if (*c == ',') ++c;
    }
  }
  const int waves = kResThreads / 64;
  const int n_ptiles = (M + 15) / 16;
  const int steps = nsteps + (has_res ? 1 : 0);
  double best = 1e30;
  for (const auto& sh : shapes) {
    const int mt = sh[0], nt = sh[1];
    const int items = ((n_ptiles + mt - 1) / mt) * ((FT + nt - 1) / nt);
    const int rounds = (items + waves - 1) / waves;
    const int simd_items = (items + 3) / 4;
    const double lds = (double)items * (nsteps * (mt * 5.6 + nt * 5.0 + 2.0) +
                                        (has_res ? mt * nt * 5.6 : 0.0) + mt * nt * 16.0 + nt * 5.0);
    const double mfma = (double)simd_items * steps * mt * nt * (mt * nt == 1 ? 24.0 : 16.0);
    const double valu = (double)simd_items * (20.0 + 9.0 * mt + nsteps * (mt + 1.0) + 8.0 * mt * nt) * 2.7;
    const double t = std::max(lds, mfma + 0.6 * valu) + rounds * 600.0;
    if (t < best) {
      best = t;
      *MT_out = mt;
      *NT_out = nt;
    }
  }
}

// A block of LDS with a lifetime in layers; blocks whose lifetimes intersect
// must not overlap.
struct LdsBlock {
  size_t units;       // 16-byte units
  int first, last;    // layers during which it is live (inclusive)
  size_t offset;
};

// Offset assignment: blocks are placed one by one at the lowest offset free
// over their whole lifetime.  The order matters; three orders are tried
// (largest first, earliest first, longest-lived first) and the tightest result
// is kept.
size_t place_in_order(std::vector<LdsBlock>& blocks, const std::vector<int>& order) {
  std::vector<int> placed;
  size_t extent = 0;
  for (int id : order) {
    LdsBlock& b = blocks[id];
    if (b.units == 0) { b.offset = 0; continue; }
    std::vector<std::pair<size_t, size_t>> busy;
    for (int other : placed) {
      const LdsBlock& o = blocks[other];
      if (o.first <= b.last && b.first <= o.last) busy.emplace_back(o.offset, o.offset + o.units);
    }
    std::sort(busy.begin(), busy.end());
    size_t at = 0;
    for (const auto& iv : busy) {
      if (at + b.units <= iv.first) break;
      at = std::max(at, iv.second);
    }
    b.offset = at;
    extent = std::max(extent, at + b.units);
    placed.push_back(id);
  }
  return extent;
}

size_t assign_offsets(std::vector<LdsBlock>& blocks) {
  std::vector<int> order(blocks.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = (int)i;
  std::vector<LdsBlock> best;
  size_t best_extent = ~size_t(0);
  for (int rule = 0; rule < 3; ++rule) {
    std::vector<int> o = order;
    std::stable_sort(o.begin(), o.end(), [&](int a, int b) {
      const LdsBlock &x = blocks[a], &y = blocks[b];
      if (rule == 0) return x.units > y.units;
      if (rule == 1) return x.first != y.first ? x.first < y.first : x.units > y.units;
      const int lx = x.last - x.first, ly = y.last - y.first;
      return lx != ly ? lx > ly : x.units > y.units;
    });
    std::vector<LdsBlock> trial = blocks;
    const size_t extent = place_in_order(trial, o);
    if (extent < best_extent) {
      best_extent = extent;
      best = trial;
    }
  }
  blocks = best;
  return best_extent;
}

// LDS pixel stride in bytes for tensors of cs 16-bit lanes.  The 16 pixels x 4
// chunks of one MFMA pixel fragment are read with one 16-byte access per lane;
// measured on gfx950 that access takes about 5 clocks of the LDS port when the
// pixel stride is an odd multiple of 32 bytes, 8.6 at other multiples of 16
// that are not multiples of 64, 8.7 at odd multiples of 64 and 16.7 at
// multiples of 128.  mode 0: the nearest odd multiple of 32; 1: the nearest
// stride that is not a multiple of 64; 2: dense.
int lds_pixel_stride(int cs, int mode) {
  const int dense = cs * 2;
  if (mode == 2) return dense;
  if (mode == 1) return dense % 64 == 0 ? dense + 16 : dense;
  int ps2 = dense;
  while (ps2 % 64 != 32) ps2 += 16;
  return ps2;
}

double lds_read_clocks(int ps2) {
  if (ps2 % 64 == 32) return 5.1;
  if (ps2 % 128 == 0) return 16.7;
  if (ps2 % 64 == 0) return 8.7;
  return 8.6;
}

// floor(v / d) = mulhi(v, reciprocal) for v < 2^16; 0 stands for d = 1
uint32_t reciprocal_u16(int d) { return d == 1 ? 0u : 0xffffffffu / (uint32_t)d + 1u; }

// Tries to lay the whole network out for resident_kernel: every per-image
// tensor (input included, final output excluded) and, for the current and the
// next layer, the tap table and the parameter blob, in LDS.
void plan_resident(fupr_model* m) {
  m->resident_ok = false;
  const int n = (int)m->ops.size();
  if (m->dt == FUPR_F32 || n > kResMaxLayers) return;
  for (const TensorInfo& t : m->tensors)
    if (t.H > 255 || t.W > 255 || t.cs > 4096) return;

  // every LDS tensor larger than 1 x 1 gets a ring of hp zero pixels
  int hp = 0;
  for (const fupr_op_desc& op : m->ops) {
    if (op.kind == FUPR_OP_CONV && (op.epilogue & (FUPR_FUSE_SCATTER | FUPR_FUSE_CAT))) return;   // per-operator kernels only
    if (op.kind == FUPR_OP_CONV) hp = std::max(hp, op.conv.pad);
    else if (op.kind != FUPR_OP_AVGPOOL) return;   // max-pool networks: images too large for LDS
  }
  for (const TensorInfo& t : m->tensors)
    if ((int64_t)(t.W + 2 * hp) * (t.H + 2 * hp) >= 65536) return;
  auto halo_of = [&](const TensorInfo& t) { return t.H * t.W > 1 ? hp : 0; };
  auto row_of = [&](const TensorInfo& t) { return t.W + 2 * halo_of(t); };

  const size_t budget_units = (kResLdsLimit - kResScratchBytes) / 16;

  // Tensors of one resolution share one pixel stride (that of the widest), so
  // that a tensor lands on the bytes of a dead tensor of the same geometry and
  // finds its halo still zero.  Per resolution the stride is the cheapest to
  // read that still lets the whole plan fit.
  struct Res { int H, W, cs, readers; };
  std::vector<Res> classes;
  std::vector<int> class_of(n + 1, -1);
  for (int tid = 0; tid <= n; ++tid) {
    const TensorInfo& t = m->tensors[tid];
    if (t.H * t.W <= 1 || tid == n) continue;
    size_t c = 0;
    while (c < classes.size() && !(classes[c].H == t.H && classes[c].W == t.W)) ++c;
    if (c == classes.size()) classes.push_back(Res{t.H, t.W, 0, 0});
    classes[c].cs = std::max(classes[c].cs, t.cs);
    class_of[tid] = (int)c;
  }
  for (const fupr_op_desc& op : m->ops)
    if (op.kind == FUPR_OP_CONV && class_of[op.in] >= 0) ++classes[class_of[op.in]].readers;
  // A block's output may be written over its shortcut tensor: the shortcut is
  // read by the lane that writes the same pixel and channels, before it writes,
  // and by nobody else; no convolution reads it in that layer.  home[t] is the
  // tensor whose LDS block t lives in.
  std::vector<int> home(n + 1);
  for (int tid = 0; tid <= n; ++tid) home[tid] = tid;
  for (int i = 0; i + 1 < n; ++i) {
    const fupr_op_desc& op = m->ops[i];
    if (op.kind != FUPR_OP_CONV || op.res < 0 || op.res == op.in) continue;
    const TensorInfo& tr = m->tensors[op.res];
    if (tr.last_use != i || op.res_spatial_stride != 1 || op.res_c_offset != 0) continue;
    if (class_of[op.res] < 0 || class_of[op.res] != class_of[i + 1]) continue;
    home[i + 1] = home[op.res];
  }
  const int k = (int)classes.size();
  std::vector<std::pair<double, std::vector<int>>> candidates;
  if (k <= 5) {
    int combos = 1;
    for (int c = 0; c < k; ++c) combos *= 3;
    for (int code = 0; code < combos; ++code) {
      std::vector<int> modes(k);
      double cost = 0.0;
      for (int c = 0, rest = code; c < k; ++c, rest /= 3) {
        modes[c] = rest % 3;
        const int ps2 = lds_pixel_stride(classes[c].cs, modes[c]);
        cost += classes[c].readers * lds_read_clocks(ps2) + 1e-6 * ps2;   // ties: the smaller stride
      }
      candidates.emplace_back(cost, modes);
    }
  } else {
    for (int mode = 0; mode < 3; ++mode) candidates.emplace_back((double)mode, std::vector<int>(k, mode));
  }
  std::stable_sort(candidates.begin(), candidates.end(),
                   [](const auto& a, const auto& b) { return a.first < b.first; });

  // Parameter blocks by size, largest first: when nothing fits with every
  // layer's parameters staged one layer ahead, the largest ones are staged at
  // the start of their own layer instead (their global-memory latency is then
  // exposed, but they need LDS for one layer only).
  std::vector<int> by_size;
  for (int i = 1; i < n; ++i)
    if (m->ops[i].kind == FUPR_OP_CONV) by_size.push_back(i);
  std::stable_sort(by_size.begin(), by_size.end(), [&](int a, int b) {
    return packed_layout(m->ops[a].conv, m->dt).total_bytes >
           packed_layout(m->ops[b].conv, m->dt).total_bytes;
  });
  for (size_t n_late = 0; n_late <= by_size.size(); ++n_late) {
  std::vector<char> late(n, 0);
  for (size_t j = 0; j < n_late; ++j) late[by_size[j]] = 1;
  for (const auto& cand : candidates) {
    std::vector<int> ps2(n + 1);
    for (int tid = 0; tid <= n; ++tid) {
      const int c = class_of[tid];
      ps2[tid] = c >= 0 ? lds_pixel_stride(classes[c].cs, cand.second[c]) : m->tensors[tid].cs * 2;
    }
    std::vector<LdsBlock> blocks(2 * (size_t)n + 1);
    for (int tid = 0; tid <= n; ++tid) {
      const TensorInfo& t = m->tensors[tid];
      LdsBlock& b = blocks[tid];
      b.first = tid - 1;                       // produced by layer tid-1 (image: before layer 0)
      b.last = std::max(t.last_use, b.first);
      b.units = tid == n ? 0 : (size_t)(t.H + 2 * halo_of(t)) * row_of(t) * ps2[tid] / 16;
      if (home[tid] != tid) {                  // written over its shortcut: that block lives on
        blocks[home[tid]].last = std::max(blocks[home[tid]].last, b.last);
        b.units = 0;
      }
    }
    bool ok = true;
    for (int i = 0; i < n && ok; ++i) {
      LdsBlock& b = blocks[n + 1 + i];
      b.first = late[i] ? i : i - 1;           // lands while layer i-1 is running, unless late
      b.last = i;
      b.units = 0;
      if (m->ops[i].kind == FUPR_OP_CONV) {
        const PackedLayout PL = packed_layout(m->ops[i].conv, m->dt);
        if (PL.nchunk_pad / 4 + kResTablePad > 64) ok = false;   // one wave stages the table
        b.units = PL.nchunk_pad / 4 + kResTablePad + PL.total_bytes / 16;   // table (16 bytes per step), blob
      }
    }
    if (!ok) return;
    const size_t extent = assign_offsets(blocks);
    if (tuning_int("debug", 0)) {
      std::fprintf(stderr, "resident candidate: strides");
      for (int c = 0; c < k; ++c)
        std::fprintf(stderr, " %dx%d:%d", classes[c].H, classes[c].W,
                     lds_pixel_stride(classes[c].cs, cand.second[c]));
      std::fprintf(stderr, " late %zu -> %zu bytes (limit %zu)\n", n_late, extent * 16,
                   budget_units * 16);
    }
    if (extent > budget_units) continue;

    // LDS byte offset of pixel (row, col) counted from the halo's corner
    auto pixel_at = [&](int tid, int row, int col) {
      const TensorInfo& t = m->tensors[tid];
      return (int32_t)(blocks[home[tid]].offset * 16 + (size_t)(row * row_of(t) + col) * ps2[tid]);
    };

    // known-zero 16-byte units, to skip re-zeroing halos that are still clean
    std::vector<uint8_t> clean(extent, 0);
    auto mark = [&](size_t first, size_t count, uint8_t v) {
      std::fill(clean.begin() + first, clean.begin() + first + count, v);
    };
    auto halo_units = [&](int tid, auto&& fn) {   // fn(unit) for every channel chunk of the halo
      const TensorInfo& t = m->tensors[tid];
      const int h = halo_of(t), Wh = row_of(t);
      for (int row = 0; row < t.H + 2 * h; ++row)
        for (int col = 0; col < Wh; ++col) {
          if (row >= h && row < t.H + h && col >= h && col < t.W + h) continue;
          const size_t u = (size_t)pixel_at(tid, row, col) / 16;
          for (int c = 0; c < t.cs / 8; ++c) fn(u + c);
        }
    };
    auto write_interior = [&](int tid) {
      const TensorInfo& t = m->tensors[tid];
      const int h = halo_of(t);
      for (int row = 0; row < t.H; ++row)
        mark((size_t)pixel_at(tid, row + h, h) / 16, (size_t)t.W * ps2[tid] / 16, 0);
    };

    ResParams& R = m->resident;
    R = ResParams{};
    const TensorInfo& t0 = m->tensors[0];
    R.in_H = t0.H;
    R.in_W = t0.W;
    R.in_Wh = row_of(t0);
    R.in_cs = t0.cs;
    R.in_ps2 = ps2[0];
    R.in_org = pixel_at(0, halo_of(t0), halo_of(t0));
    R.hp = hp;
    R.lds_bytes = (int)(kResScratchBytes + extent * 16);
    R.out_pixels = m->tensors[n].H * m->tensors[n].W;
    write_interior(0);
    halo_units(0, [&](size_t u) { clean[u] = 1; });
    if (blocks[n + 1].units) mark(blocks[n + 1].offset, blocks[n + 1].units, 0);

    std::array<int, 8> prev_geometry;
    prev_geometry.fill(-1);
    m->res_layers.clear();
    m->res_tables.clear();
    m->res_table_at.clear();
    for (int i = 0; i < n; ++i) {
      const fupr_op_desc& op = m->ops[i];
      const TensorInfo& ti = m->tensors[op.in];
      const TensorInfo& to = m->tensors[i + 1];
      const bool last = i + 1 == n;
      ResLayer L{};
      size_t table_at = 0;
      L.flags = last ? kResLast : 0;
      if (late[i]) {
        // an entry that does nothing but stage this layer's parameters
        ResLayer stage{};
        stage.res_org = -1;
        stage.MT = stage.NT = stage.n_fgroups = stage.Q = stage.M = 1;   // a conv entry without work items
        m->res_layers.push_back(stage);
        m->res_table_at.push_back(0);
        if (blocks[n + 1 + i].units) mark(blocks[n + 1 + i].offset, blocks[n + 1 + i].units, 0);
      }
      L.res_org = -1;
      L.out_org = last ? 0 : pixel_at(i + 1, halo_of(to), halo_of(to));
      L.cs_out = to.cs;
      L.M = to.H * to.W;
      L.Q = to.W;
      L.MT = L.NT = L.n_fgroups = 1;
      if (op.kind == FUPR_OP_AVGPOOL) {
        L.flags |= kResMean;
        L.in_org = pixel_at(op.in, halo_of(ti), halo_of(ti));
        L.in_row = row_of(ti) * ps2[op.in];
        L.in_col = ps2[op.in];
        L.M = ti.H * ti.W;       // the mean layer iterates over its INPUT extent
        L.Q = ti.W;
        // partial sums held in the scratch area: MT parts x cs_out floats
        L.MT = std::min(8, kResScratchBytes / 4 / to.cs);
        if (L.MT < 1 || L.MT * to.cs > kResThreads) return;
      } else {
        const fupr_conv_shape& s = op.conv;
        const PackedLayout PL = packed_layout(s, m->dt);
        if (halo_of(ti) < s.pad) return;   // a padded conv on a 1 x 1 image: not laid out here
        const int nsteps = PL.nchunk_pad / 4, cpt = PL.Cp / 8;
        L.packed = op.packed;
        L.blob_units = (int32_t)(PL.total_bytes / 16);
        L.tab_units = nsteps + kResTablePad;
        L.tab_off = (int32_t)(blocks[n + 1 + i].offset * 16);
        L.w_off = L.tab_off + L.tab_units * 16;
        L.wts_off = L.w_off + (int32_t)PL.weight_offset;
        L.wstep = 4 * PL.Kp * 16;
        L.in_org = pixel_at(op.in, halo_of(ti) - s.pad, halo_of(ti) - s.pad);
        L.in_row = s.stride * row_of(ti) * ps2[op.in];
        L.in_col = s.stride * ps2[op.in];
        L.out_row = row_of(to) * ps2[i + 1];
        L.out_col = ps2[i + 1];
        L.nsteps = nsteps;
        L.FT = PL.Kp / 16;
        if (op.epilogue & FUPR_FUSE_RELU) L.flags |= kResRelu;
        if (op.res >= 0) {
          if (op.res_c_offset != 0) return;
          const TensorInfo& tr = m->tensors[op.res];
          L.res_org = pixel_at(op.res, halo_of(tr), halo_of(tr));
          L.res_cs = tr.cs;
          L.res_row = op.res_spatial_stride * row_of(tr) * ps2[op.res];
          L.res_col = op.res_spatial_stride * ps2[op.res];
        }
        int mt = 1, nt = 1;
        resident_item_shape(L.M, L.FT, nsteps, op.res >= 0, &mt, &nt);
        L.MT = mt;
        L.NT = nt;
        L.n_fgroups = (L.FT + nt - 1) / nt;
        L.n_items = ((L.M + 15) / 16 + mt - 1) / mt * L.n_fgroups;
        if (L.n_items >= 65536) return;
        if (L.M % (16 * mt) == 0) L.flags |= kResFullPixels;
        if (L.FT % nt == 0 && to.cs == PL.Kp && !last) L.flags |= kResFullFilters;
        if (op.res >= 0 && L.res_row == L.out_row && L.res_col == L.out_col) L.flags |= kResLikeOut;
        const std::array<int, 8> geometry = {L.M, L.Q, mt, L.n_fgroups, L.in_row, L.in_col, L.out_row, L.out_col};
        if (L.n_items <= kResThreads / 64) {
          if (geometry == prev_geometry && (L.flags & kResFullPixels) && !last && L.in_row == L.out_row &&
              L.in_col == L.out_col)
            L.flags |= kResReuse;
          prev_geometry = geometry;
        } else {
          prev_geometry.fill(-1);   // later work items overwrite what the first one left
        }
        // tap table: LDS byte offset of every chunk of output pixel (0, 0)'s
        // window; padding chunks (zero weights) and the padding steps after the
        // last one re-read the first chunk: finite data
        table_at = m->res_tables.size();
        for (int j = 0; j < L.tab_units * 4; ++j) {
          int32_t e = 0;
          if (j < PL.nchunk) {
            const int tap = j / cpt, c8 = j - tap * cpt;
            const int r = tap / s.S, sx = tap - r * s.S;
            e = (r * row_of(ti) + sx) * ps2[op.in] + c8 * 16;
          }
          m->res_tables.push_back(L.in_org + e);
        }
      }
      L.magicQ = reciprocal_u16(L.Q);
      L.magicF = reciprocal_u16(L.n_fgroups);
      if (!last) {
        bool dirty = false;
        halo_units(i + 1, [&](size_t u) { dirty = dirty || !clean[u]; });
        if (dirty) {
          L.flags |= kResZeroHalo;
          L.hz_org = L.out_org;
          L.hz_P = to.H;
          L.hz_Q = to.W;
          L.hz_Wh = row_of(to);
          L.hz_ps2 = ps2[i + 1];
          L.hz_chunks = to.cs / 8;
          L.hz_hp = halo_of(to);
          halo_units(i + 1, [&](size_t u) { clean[u] = 1; });
        }
        if (halo_of(to) > 0) write_interior(i + 1);
        else mark(blocks[home[i + 1]].offset, blocks[home[i + 1]].units, 0);
      }
      if (i + 1 < n && !late[i + 1] && blocks[n + 2 + i].units)
        mark(blocks[n + 2 + i].offset, blocks[n + 2 + i].units, 0);
      m->res_layers.push_back(L);
      m->res_table_at.push_back(table_at);
      if (tuning_int("debug", 0))
        std::fprintf(stderr, "resident layer %d: M %d FT %d steps %d item %dx%d items %d ps2 in %d out %d "
                     "zero_halo %d res %d\n", i, L.M, L.FT, L.nsteps, L.MT, L.NT, L.n_items, ps2[op.in],
                     ps2[i + 1], (L.flags & kResZeroHalo) != 0, L.res_org >= 0);
    }
    if (m->res_layers.size() > (size_t)kResMaxLayers) return;
    R.n_layers = (int)m->res_layers.size();
    if (tuning_int("debug", 0))
      std::fprintf(stderr, "resident plan: %d bytes of LDS, %d table entries for %d layers\n",
                   R.lds_bytes, R.n_layers, n);
    m->resident_ok = true;
    return;
  }
  }
}

void release_side(fupr_model* m);   // below, with the forked schedule
bool conv_conv_pair(const fupr_model* m, size_t i);   // below, with the launch list

// Sizes of the one-kernel schedule's table: the layer entries, then the tap tables.
size_t resident_layer_bytes(const fupr_model* m) {
  return round_up_sz(m->res_layers.size() * sizeof(ResLayer), 256);
}
size_t resident_table_bytes(const fupr_model* m) {
  return round_up_sz(m->res_tables.size() * sizeof(int32_t), 256) + 256;
}

}  // namespace

extern "C" fupr_status fupr_model_create(const fupr_graph_desc* g, fupr_model** out) {
  if (!g || !out || !g->ops) return FUPR_ERR_NULL;
  if (!dtype_ok((int)g->dt)) return FUPR_ERR_DTYPE;
  if (g->n_ops <= 0 || g->C <= 0 || g->H <= 0 || g->W <= 0) return FUPR_ERR_SHAPE;

  fupr_model* m = new (std::nothrow) fupr_model;
  if (!m) return FUPR_ERR_ARG;
  m->dt = g->dt;
  m->ops.assign(g->ops, g->ops + g->n_ops);
  m->tensors.resize(g->n_ops + 1);
  m->tensors[0] = TensorInfo{g->C, g->H, g->W, min_c_stride(g->C, g->dt), -1, -1};

  fupr_status err = FUPR_OK;
  for (int i = 0; i < g->n_ops && err == FUPR_OK; ++i) {
    const fupr_op_desc& op = m->ops[i];
    if (op.in < 0 || op.in > i) { err = FUPR_ERR_ARG; break; }
    const TensorInfo& tin = m->tensors[op.in];
    TensorInfo t{};
    t.buffer = -3;
    t.last_use = -1;
    if (op.kind == FUPR_OP_CONV) {
      const fupr_conv_shape& s = op.conv;
      if (!shape_ok(&s)) { err = FUPR_ERR_SHAPE; break; }
      if (!op.packed) { err = FUPR_ERR_NULL; break; }
      if (op.epilogue & ~uint32_t(FUPR_FUSE_RELU | FUPR_FUSE_ADD | FUPR_FUSE_SCATTER | FUPR_FUSE_CAT)) {
        err = FUPR_ERR_ARG; break;
      }
      const bool cat = (op.epilogue & FUPR_FUSE_CAT) != 0;
      int c_in = tin.C;
      if (cat) {
        // a 1 x 1 convolution over tensor `in` and tensor `in2` concatenated along the channels
        if (g->dt == FUPR_F32) { err = FUPR_ERR_DTYPE; break; }
        if (op.in2 < 0 || op.in2 > i || (op.in2_spatial_stride != 1 && op.in2_spatial_stride != 2) ||
            (op.epilogue & FUPR_FUSE_SCATTER)) {
          err = FUPR_ERR_ARG; break;
        }
        const TensorInfo& t2 = m->tensors[op.in2];
        if (s.R != 1 || s.S != 1 || s.stride != 1 || s.pad != 0 ||
            (int64_t)(tin.H - 1) * op.in2_spatial_stride >= t2.H ||
            (int64_t)(tin.W - 1) * op.in2_spatial_stride >= t2.W) {
          err = FUPR_ERR_SHAPE; break;
        }
        c_in = round_up(tin.C, FUPR_CAT_ALIGN) + t2.C;
      }
      if (s.C != c_in || tin.H + 2 * s.pad < s.R || tin.W + 2 * s.pad < s.S) {
        err = FUPR_ERR_SHAPE; break;
      }
      const bool scatter = (op.epilogue & FUPR_FUSE_SCATTER) != 0;
      if (scatter != (op.keep_idx != nullptr)) { err = scatter ? FUPR_ERR_NULL : FUPR_ERR_ARG; break; }
      t.C = s.K;
      t.H = out_extent(tin.H, s.R, s.stride, s.pad);
      t.W = out_extent(tin.W, s.S, s.stride, s.pad);
      const bool add = (op.epilogue & FUPR_FUSE_ADD) != 0;
      if (add != (op.res >= 0)) { err = FUPR_ERR_ARG; break; }
      if (add) {
        if (op.res > i) { err = FUPR_ERR_ARG; break; }
        const TensorInfo& tr = m->tensors[op.res];
        if (op.res_spatial_stride < 1 || op.res_c_offset < 0 || op.res_c_offset % 4 != 0) {
          err = FUPR_ERR_ARG; break;
        }
        if (scatter) {
          // the kept output filters add into tensor res in place; the output is that tensor
          if (g->dt == FUPR_F32) { err = FUPR_ERR_DTYPE; break; }
          if (op.res == 0 || i + 1 == g->n_ops || op.res_spatial_stride != 1 || op.res_c_offset != 0 ||
              op.res == op.in) {
            err = FUPR_ERR_ARG; break;
          }
          if (s.K > tr.C || tr.H != t.H || tr.W != t.W) { err = FUPR_ERR_SHAPE; break; }
          t.C = tr.C;
        } else if (op.res_c_offset + tr.C > s.K ||
                   (int64_t)(t.H - 1) * op.res_spatial_stride >= tr.H ||
                   (int64_t)(t.W - 1) * op.res_spatial_stride >= tr.W) {
          err = FUPR_ERR_SHAPE; break;
        }
      } else if (scatter) {
        err = FUPR_ERR_ARG; break;
      }
    } else if (op.kind == FUPR_OP_MAXPOOL) {
      const int k = op.conv.R;
      if (k <= 0 || op.conv.S != k || op.conv.stride <= 0 || op.conv.pad < 0 || op.conv.pad >= k) {
        err = FUPR_ERR_ARG; break;
      }
      if (op.res >= 0) { err = FUPR_ERR_ARG; break; }
      if (tin.H + 2 * op.conv.pad < k || tin.W + 2 * op.conv.pad < k) { err = FUPR_ERR_SHAPE; break; }
      t.C = tin.C;
      t.H = out_extent(tin.H, k, op.conv.stride, op.conv.pad);
      t.W = out_extent(tin.W, k, op.conv.stride, op.conv.pad);
    } else if (op.kind == FUPR_OP_AVGPOOL) {
      if (op.res >= 0) { err = FUPR_ERR_ARG; break; }
      t.C = tin.C;
      t.H = 1;
      t.W = 1;
    } else {
      err = FUPR_ERR_ARG; break;
    }
    t.cs = min_c_stride(t.C, g->dt);
    m->tensors[i + 1] = t;
  }
  if (err != FUPR_OK) {
    delete m;
    return err;
  }

  // Liveness and greedy buffer sharing.
  const int n = g->n_ops;
  for (int i = 0; i < n; ++i) {
    m->tensors[m->ops[i].in].last_use = i;
    if (m->ops[i].res >= 0) m->tensors[m->ops[i].res].last_use = i;
    if (m->ops[i].kind == FUPR_OP_CONV && (m->ops[i].epilogue & FUPR_FUSE_CAT))
      m->tensors[m->ops[i].in2].last_use = i;
  }
  // a tensor updated in place must have no reader after the update
  for (int i = 0; i < n; ++i) {
    if (!(m->ops[i].epilogue & FUPR_FUSE_SCATTER) || m->ops[i].kind != FUPR_OP_CONV) continue;
    if (m->tensors[m->ops[i].res].last_use != i) {
      delete m;
      return FUPR_ERR_ARG;
    }
  }
  // two convolutions that may run as one kernel: what the first reads must
  // outlive the second, whose output is written while the first still reads
  for (int i = 0; i + 1 < n; ++i) {
    if (!conv_conv_pair(m, (size_t)i)) continue;
    TensorInfo& tin = m->tensors[m->ops[i].in];
    tin.last_use = std::max(tin.last_use, i + 1);
    if (m->ops[i].res >= 0) {
      TensorInfo& tr = m->tensors[m->ops[i].res];
      tr.last_use = std::max(tr.last_use, i + 1);
    }
    if (m->ops[i].epilogue & FUPR_FUSE_CAT) {
      TensorInfo& t2 = m->tensors[m->ops[i].in2];
      t2.last_use = std::max(t2.last_use, i + 1);
    }
  }
  std::vector<int> holder;  // buffer -> tensor id it holds, -1 = free
  for (int i = 0; i < n; ++i) {
    const int tid = i + 1;
    TensorInfo& t = m->tensors[tid];
    if (tid == n) {
      t.buffer = -2;
    } else if (m->ops[i].kind == FUPR_OP_CONV && (m->ops[i].epilogue & FUPR_FUSE_SCATTER)) {
      // the operator's output is the tensor it updated: same buffer, new holder
      t.buffer = m->tensors[m->ops[i].res].buffer;
      holder[t.buffer] = tid;
    } else {
      const size_t need = (size_t)t.H * t.W * t.cs;
      int pick = -1;
      for (size_t b = 0; b < holder.size(); ++b) {
        if (holder[b] >= 0) continue;
        // prefer the free buffer whose size is closest to what is needed
        if (pick < 0) pick = (int)b;
        else {
          const size_t cur = m->buffer_elems[pick], cand = m->buffer_elems[b];
          const size_t dc = cur > need ? cur - need : need - cur;
          const size_t dn = cand > need ? cand - need : need - cand;
          if (dn < dc) pick = (int)b;
        }
      }
      if (pick < 0) {
        holder.push_back(-1);
        m->buffer_elems.push_back(0);
        pick = (int)holder.size() - 1;
      }
      holder[pick] = tid;
      m->buffer_elems[pick] = std::max(m->buffer_elems[pick], need);
      t.buffer = pick;
    }
    // tensors whose last reader is this operator become free afterwards
    for (size_t b = 0; b < holder.size(); ++b) {
      const int h = holder[b];
      if (h >= 0 && h != tid && m->tensors[h].last_use <= i) holder[b] = -1;
    }
  }
  plan_resident(m);
  *out = m;
  return FUPR_OK;
}

extern "C" fupr_status fupr_model_set_schedule(fupr_model* m, int32_t schedule) {
  if (!m) return FUPR_ERR_NULL;
  if (schedule != FUPR_SCHEDULE_AUTO && schedule != FUPR_SCHEDULE_PER_LAYER) return FUPR_ERR_ARG;
  m->schedule = schedule;
  return FUPR_OK;
}

extern "C" size_t fupr_model_table_bytes(const fupr_model* m) {
  if (!m || !m->resident_ok) return 0;
  return resident_layer_bytes(m) + resident_table_bytes(m);
}

extern "C" fupr_status fupr_model_table_write(const fupr_model* m, const void* dev_table,
                                              void* host_out) {
  if (!m || !dev_table || !host_out) return FUPR_ERR_NULL;
  if (!m->resident_ok) return FUPR_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(dev_table) & 255u) != 0) return FUPR_ERR_ALIGN;
  const size_t n = m->res_layers.size();
  const size_t layer_bytes = resident_layer_bytes(m);
  const char* base = reinterpret_cast<const char*>(dev_table);
  std::vector<ResLayer> layers = m->res_layers;
  for (size_t i = 0; i < n; ++i)
    layers[i].table = base + layer_bytes + m->res_table_at[i] * sizeof(int32_t);
  for (size_t i = 0; i + 1 < n; ++i) {
    layers[i].next_packed = layers[i + 1].packed;
    layers[i].next_table = layers[i + 1].table;
    layers[i].next_blob_units = layers[i + 1].blob_units;
    layers[i].next_tab_units = layers[i + 1].tab_units;
    layers[i].next_w_off = layers[i + 1].w_off;
    layers[i].next_tab_off = layers[i + 1].tab_off;
  }
  char* out = reinterpret_cast<char*>(host_out);
  std::fill(out, out + layer_bytes + resident_table_bytes(m), 0);
  std::copy(reinterpret_cast<const char*>(layers.data()),
            reinterpret_cast<const char*>(layers.data()) + n * sizeof(ResLayer), out);
  std::copy(reinterpret_cast<const char*>(m->res_tables.data()),
            reinterpret_cast<const char*>(m->res_tables.data()) + m->res_tables.size() * sizeof(int32_t),
            out + layer_bytes);
  return FUPR_OK;
}

extern "C" fupr_status fupr_model_set_table(fupr_model* m, const void* dev_table) {
  if (!m) return FUPR_ERR_NULL;
  if (dev_table && !m->resident_ok) return FUPR_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(dev_table) & 255u) != 0) return FUPR_ERR_ALIGN;
  m->res_dev = dev_table;
  return FUPR_OK;
}

extern "C" fupr_status fupr_model_set_side_streams(fupr_model* m, int32_t n, void* const* streams) {
  if (!m || (n > 0 && !streams)) return FUPR_ERR_NULL;
  if (n < 0 || n > kMaxSplit - 1) return FUPR_ERR_ARG;
  for (int k = 0; k < n; ++k)
    if (!streams[k]) return FUPR_ERR_NULL;   // the default stream cannot be forked into a capture
  std::lock_guard<std::mutex> lock(m->side_mutex);
  release_side(m);
  if (n == 0) return FUPR_OK;
  bool ok = hipEventCreateWithFlags(&m->fork_event, hipEventDisableTiming) == hipSuccess;
  for (int k = 0; ok && k < n; ++k)
    ok = hipEventCreateWithFlags(&m->join_event[k], hipEventDisableTiming) == hipSuccess;
  if (!ok) {
    (void)hipGetLastError();
    release_side(m);
    return FUPR_ERR_LAUNCH;
  }
  for (int k = 0; k < n; ++k) m->side_stream[k] = reinterpret_cast<hipStream_t>(streams[k]);
  m->n_side = n;
  return FUPR_OK;
}

extern "C" void fupr_model_destroy(fupr_model* m) {
  if (!m) return;
  release_side(m);
  delete m;
}

extern "C" int32_t fupr_model_num_ops(const fupr_model* m) { return m ? (int32_t)m->ops.size() : 0; }

extern "C" size_t fupr_model_workspace_bytes(const fupr_model* m, int32_t batch) {
  if (!m || batch <= 0) return 0;
  size_t total = 0;
  for (size_t e : m->buffer_elems) total += round_up_sz(e * (size_t)batch * elem_size(m->dt), 256);
  return std::max<size_t>(total, 256);
}

extern "C" fupr_status fupr_model_output_shape(const fupr_model* m, int32_t batch,
                                               fupr_tensor* out) {
  if (!m || !out) return FUPR_ERR_NULL;
  if (batch <= 0) return FUPR_ERR_SHAPE;
  const TensorInfo& t = m->tensors.back();
  out->N = batch;
  out->H = t.H;
  out->W = t.W;
  out->C = t.C;
  out->c_stride = t.cs;
  out->dt = m->dt;
  out->ptr = nullptr;
  return FUPR_OK;
}

namespace {

// The one-kernel schedule applies when the plan exists, the caller has not
// asked for per-layer kernels, and the caller's tensors have the strides the
// plan assumed.
bool use_resident(const fupr_model* m, const fupr_tensor* input, const fupr_tensor* output) {
  if (!m->resident_ok || !m->res_dev || m->schedule != FUPR_SCHEDULE_AUTO) return false;
  if (input->c_stride != m->tensors.front().cs) return false;
  const fupr_op_desc& last = m->ops.back();
  const int limit = last.kind == FUPR_OP_CONV ? round_up(last.conv.K, 16) : m->tensors[last.in].cs;
  return output->c_stride <= limit;
}

// One kernel launch of the per-operator schedule: `count` consecutive operators.
struct Launch {
  int first, count;
};

// Operator i is a 16-bit 7 x 7 stem convolution with ReLU whose only reader is
// the 3 x 3 max-pool right behind it: the two run as one kernel.
bool stem_pool_pair(const fupr_model* m, size_t i) {
  if (m->schedule != FUPR_SCHEDULE_AUTO || i + 1 >= m->ops.size()) return false;
  const fupr_op_desc& c = m->ops[i];
  const fupr_op_desc& q = m->ops[i + 1];
  if (c.kind != FUPR_OP_CONV || c.res >= 0 || c.epilogue != FUPR_FUSE_RELU) return false;
  if (q.kind != FUPR_OP_MAXPOOL || q.in != (int)i + 1) return false;
  if (m->tensors[i + 1].last_use != (int)i + 1) return false;
  const TensorInfo& tin = m->tensors[c.in];
  return stem_pool_applies(c.conv, m->dt, 1, tin.H, tin.W, tin.cs, m->tensors[i + 2].cs, q.conv.R,
                           q.conv.stride, q.conv.pad);
}

// Operator i is a 1 x 1 convolution whose whole output tile a wave holds, and
// operator i + 1 a 1 x 1 convolution of exactly that tensor (a bottleneck
// block's last convolution and the next block's first): one kernel computes
// both, the second from the first one's registers.
bool conv_conv_pair(const fupr_model* m, size_t i) {
  if (m->schedule != FUPR_SCHEDULE_AUTO || i + 1 >= m->ops.size()) return false;
  const fupr_op_desc& a = m->ops[i];
  const fupr_op_desc& b = m->ops[i + 1];
  if (a.kind != FUPR_OP_CONV || b.kind != FUPR_OP_CONV) return false;
  if ((a.epilogue | b.epilogue) & FUPR_FUSE_SCATTER) return false;
  if (b.epilogue & FUPR_FUSE_CAT) return false;
  if ((a.epilogue & FUPR_FUSE_CAT) && a.res >= 0) return false;
  if (b.in != (int)i + 1 || b.res >= 0) return false;
  const TensorInfo& tin = m->tensors[a.in];
  return conv_pair_fusable(a.conv, b.conv, m->dt, 1, tin.H, tin.W);
}

std::vector<Launch> launches_of(const fupr_model* m) {
  std::vector<Launch> v;
  for (size_t i = 0; i < m->ops.size();) {
    const int count = (stem_pool_pair(m, i) || conv_conv_pair(m, i)) ? 2 : 1;
    v.push_back(Launch{(int)i, count});
    i += count;
  }
  return v;
}

// Sub-batches of the per-operator schedule.  Two sub-batches side by side let one's
// memory-bound kernels run beside the other's arithmetic and fill launch gaps and tails.
// Measured on the ImageNet-size workloads (one / two / three / four sub-batches): the
// bottleneck network, whose 1 x 1 convolutions move 75 - 100 flops per byte, 3261 / 2988 /
// 3220 / 3320 us at 256 images and 922 / 888 / 960 / 1058 us at 64; the basic-block network
// (258 flops per byte, kernels that fill the compute units only at full batch) 417 / 448 us
// at 64.  So: two sub-batches from 192 images on, and from 64 images on for networks under
// 150 flops per byte; else one; never more than the caller has lent streams for.  The
// tuning switch split=<1..4> forces a count.
int split_count(const fupr_model* m, int N) {
  const int forced = std::min(std::max(tuning_int("split", 0), 0), kMaxSplit);
  int want = forced ? std::min(forced, std::max(N / 8, 1)) : (N >= 192 ? 2 : 1);
  if (!forced && want == 1 && N >= 64 && m->n_side > 0) {
    double flops = 0.0, bytes = 0.0;
    for (int32_t i = 0; i < (int32_t)m->ops.size(); ++i) {
      fupr_op_stats s;
      if (fupr_model_op_stats(m, N, i, &s) != FUPR_OK) return 1;
      flops += s.flops;
      bytes += s.bytes;
    }
    if (bytes > 0.0 && flops / bytes < 150.0) want = 2;
  }
  return std::min(want, m->n_side + 1);
}

void release_side(fupr_model* m) {
  if (m->fork_event) (void)hipEventDestroy(m->fork_event);
  m->fork_event = nullptr;
  for (int k = 0; k < kMaxSplit - 1; ++k) {
    if (m->join_event[k]) (void)hipEventDestroy(m->join_event[k]);
    m->join_event[k] = nullptr;
    m->side_stream[k] = nullptr;
  }
  m->n_side = 0;
}

fupr_status run(const fupr_model* m, const fupr_tensor* input, const fupr_tensor* output,
                void* workspace, size_t workspace_bytes, void* stream, hipEvent_t* events) {
  if (!m || !input || !output || !workspace) return FUPR_ERR_NULL;
  if (!input->ptr || !output->ptr) return FUPR_ERR_NULL;
  if (input->dt != m->dt || output->dt != m->dt) return FUPR_ERR_DTYPE;
  const TensorInfo& t0 = m->tensors.front();
  const TensorInfo& tl = m->tensors.back();
  const int N = input->N;
  if (N <= 0 || input->C != t0.C || input->H != t0.H || input->W != t0.W) return FUPR_ERR_SHAPE;
  if (output->N != N || output->C != tl.C || output->H != tl.H || output->W != tl.W)
    return FUPR_ERR_SHAPE;
  if (input->c_stride < t0.C || input->c_stride % c_align(m->dt) != 0) return FUPR_ERR_ALIGN;
  if (output->c_stride < tl.C || output->c_stride % c_align(m->dt) != 0) return FUPR_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return FUPR_ERR_WORKSPACE;
  if (workspace_bytes < fupr_model_workspace_bytes(m, N)) return FUPR_ERR_WORKSPACE;
  for (const TensorInfo& t : m->tensors)
    if ((int64_t)N * t.H * t.W * t.cs >= (int64_t(1) << 31)) return FUPR_ERR_LIMIT;

  std::vector<char*> base(m->buffer_elems.size());
  size_t off = 0;
  for (size_t b = 0; b < base.size(); ++b) {
    base[b] = reinterpret_cast<char*>(workspace) + off;
    off += round_up_sz(m->buffer_elems[b] * (size_t)N * elem_size(m->dt), 256);
  }
  // images n0 .. n0 + count - 1 of a tensor; inside a workspace buffer every
  // sub-batch owns the slice its images would need at the buffer's largest tensor
  const size_t es = elem_size(m->dt);
  auto view = [&](int tid, int n0, int count) {
    const TensorInfo& t = m->tensors[tid];
    fupr_tensor v;
    v.N = count; v.H = t.H; v.W = t.W; v.C = t.C; v.dt = m->dt;
    char* ptr;
    if (t.buffer == -1) {
      v.c_stride = input->c_stride;
      ptr = (char*)input->ptr + (size_t)n0 * t.H * t.W * input->c_stride * es;
    } else if (t.buffer == -2) {
      v.c_stride = output->c_stride;
      ptr = (char*)output->ptr + (size_t)n0 * t.H * t.W * output->c_stride * es;
    } else {
      v.c_stride = t.cs;
      ptr = base[t.buffer] + (size_t)n0 * m->buffer_elems[t.buffer] * es;
    }
    v.ptr = ptr;
    return v;
  };

  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  if (events && hipEventRecord(events[0], hs) != hipSuccess) return FUPR_ERR_LAUNCH;
  if (use_resident(m, input, output)) {
    ResParams R = m->resident;
    R.layers = reinterpret_cast<const ResLayer*>(m->res_dev);
    R.x = input->ptr;
    R.y = output->ptr;
    R.y_cs = output->c_stride;
    const fupr_status st = launch_resident(R, N, m->dt, stream);
    if (st != FUPR_OK) return st;
    if (events && hipEventRecord(events[1], hs) != hipSuccess) return FUPR_ERR_LAUNCH;
    return FUPR_OK;
  }
  const std::vector<Launch> launches = launches_of(m);
  auto enqueue = [&](int n0, int count, void* on, bool record) -> fupr_status {
    for (size_t l = 0; l < launches.size(); ++l) {
      const size_t i = (size_t)launches[l].first;
      const fupr_op_desc& op = m->ops[i];
      const fupr_tensor x = view(op.in, n0, count);
      const fupr_tensor y = view((int)i + launches[l].count, n0, count);
      fupr_status st;
      if (launches[l].count == 2 && m->ops[i + 1].kind == FUPR_OP_CONV) {
        const fupr_op_desc& second = m->ops[i + 1];
        const fupr_tensor mid = view((int)i + 1, n0, count);
        fupr_residual r;
        const bool add = op.res >= 0;
        if (add) {
          r.t = view(op.res, n0, count);
          r.spatial_stride = op.res_spatial_stride;
          r.c_offset = op.res_c_offset;
        }
        if (op.epilogue & FUPR_FUSE_CAT) {
          const fupr_tensor x2 = view(op.in2, n0, count);
          st = conv_cat_conv1x1_fused(&op.conv, &x, &x2, op.in2_spatial_stride, op.packed,
                                      op.epilogue & ~uint32_t(FUPR_FUSE_CAT), &mid, &second.conv,
                                      second.packed, second.epilogue, &y, on);
        } else {
          st = fupr_conv_conv1x1_fused(&op.conv, &x, op.packed, add ? &r : nullptr, op.epilogue, &mid,
                                       &second.conv, second.packed, second.epilogue, &y, on);
        }
      } else if (launches[l].count == 2) {
        const fupr_op_desc& pool = m->ops[i + 1];
        st = fupr_conv_maxpool_fused(&op.conv, &x, op.packed, pool.conv.R, pool.conv.stride,
                                     pool.conv.pad, &y, on);
      } else if (op.kind == FUPR_OP_CONV && (op.epilogue & FUPR_FUSE_SCATTER)) {
        st = fupr_conv_scatter_fused(&op.conv, &x, op.packed, op.keep_idx,
                                     op.epilogue & FUPR_FUSE_RELU, &y, on);
      } else if (op.kind == FUPR_OP_CONV) {
        fupr_residual r;
        const bool add = op.res >= 0;
        if (add) {
          r.t = view(op.res, n0, count);
          r.spatial_stride = op.res_spatial_stride;
          r.c_offset = op.res_c_offset;
        }
        if (op.epilogue & FUPR_FUSE_CAT) {
          const fupr_tensor x2 = view(op.in2, n0, count);
          st = fupr_conv_cat_fused(&op.conv, &x, &x2, op.in2_spatial_stride, op.packed,
                                   add ? &r : nullptr, op.epilogue & ~uint32_t(FUPR_FUSE_CAT), &y, on);
        } else {
          st = fupr_conv_fused(&op.conv, &x, op.packed, add ? &r : nullptr, op.epilogue, &y, on);
        }
      } else if (op.kind == FUPR_OP_MAXPOOL) {
        st = fupr_maxpool(&x, op.conv.R, op.conv.stride, op.conv.pad, &y, on);
      } else {
        st = fupr_global_avgpool(&x, &y, on);
      }
      if (st != FUPR_OK) return st;
      if (record && hipEventRecord(events[l + 1], hs) != hipSuccess) return FUPR_ERR_LAUNCH;
    }
    return FUPR_OK;
  };
  // Timed runs and small batches stay on the caller's stream; otherwise the
  // batch is cut into sub-batches that run side by side (images are independent).
  const int split = events || m->schedule != FUPR_SCHEDULE_AUTO ? 1 : split_count(m, N);
  if (split <= 1) return enqueue(0, N, stream, events != nullptr);
  std::lock_guard<std::mutex> lock(const_cast<fupr_model*>(m)->side_mutex);
  if (hipEventRecord(m->fork_event, hs) != hipSuccess) return FUPR_ERR_LAUNCH;
  fupr_status result = FUPR_OK;
  int forked = 0;   // side streams that wait on the caller's stream and must be joined to it again
  for (int k = 1; k < split && result == FUPR_OK; ++k) {
    if (hipStreamWaitEvent(m->side_stream[k - 1], m->fork_event, 0) != hipSuccess) result = FUPR_ERR_LAUNCH;
    else ++forked;
  }
  for (int k = 0; k < split && result == FUPR_OK; ++k) {
    const int n0 = (int)((int64_t)N * k / split), n1 = (int)((int64_t)N * (k + 1) / split);
    result = enqueue(n0, n1 - n0, k == 0 ? stream : (void*)m->side_stream[k - 1], false);
  }
  // always join what was forked, so that the caller's stream (or capture) is whole again
  for (int k = 1; k <= forked; ++k) {
    if (hipEventRecord(m->join_event[k - 1], m->side_stream[k - 1]) != hipSuccess ||
        hipStreamWaitEvent(hs, m->join_event[k - 1], 0) != hipSuccess)
      result = FUPR_ERR_LAUNCH;
  }
  return result;
}

}  // namespace

extern "C" fupr_status fupr_forward(const fupr_model* m, const fupr_tensor* input,
                                    const fupr_tensor* output, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  return run(m, input, output, workspace, workspace_bytes, stream, nullptr);
}

extern "C" fupr_status fupr_forward_timed(const fupr_model* m, const fupr_tensor* input,
                                          const fupr_tensor* output, void* workspace,
                                          size_t workspace_bytes, void* stream, float* op_ms) {
  if (!m || !op_ms) return FUPR_ERR_NULL;
  const size_t n = m->ops.size();
  std::vector<hipEvent_t> ev(n + 1, nullptr);
  fupr_status st = FUPR_OK;
  for (size_t i = 0; i <= n; ++i)
    if (hipEventCreate(&ev[i]) != hipSuccess) { st = FUPR_ERR_LAUNCH; break; }
  if (st == FUPR_OK) st = run(m, input, output, workspace, workspace_bytes, stream, ev.data());
  if (st == FUPR_OK && hipStreamSynchronize(reinterpret_cast<hipStream_t>(stream)) != hipSuccess)
    st = FUPR_ERR_LAUNCH;
  if (st == FUPR_OK) {
    std::vector<float> ms(n, 0.0f);
    const size_t launches = use_resident(m, input, output) ? 1 : launches_of(m).size();
    for (size_t i = 0; i < launches; ++i)
      if (hipEventElapsedTime(&ms[i], ev[i], ev[i + 1]) != hipSuccess) { st = FUPR_ERR_LAUNCH; break; }
    if (st == FUPR_OK) std::copy(ms.begin(), ms.end(), op_ms);
  }
  for (hipEvent_t e : ev)
    if (e) (void)hipEventDestroy(e);
  return st;
}

extern "C" fupr_status fupr_model_op_stats(const fupr_model* m, int32_t batch, int32_t op,
                                           fupr_op_stats* out) {
  if (!m || !out) return FUPR_ERR_NULL;
  if (batch <= 0 || op < 0 || op >= (int32_t)m->ops.size()) return FUPR_ERR_ARG;
  const fupr_op_desc& d = m->ops[op];
  const TensorInfo& ti = m->tensors[d.in];
  const TensorInfo& to = m->tensors[op + 1];
  const double es = (double)elem_size(m->dt);
  fupr_op_stats s{};
  s.first_op = op;
  s.n_ops = 1;
  s.M = (int64_t)batch * to.H * to.W;
  s.K = to.C;
  s.C = ti.C;
  const double in_b = es * batch * (double)ti.H * ti.W * ti.C;
  const double out_b = es * (double)s.M * to.C;
  if (d.kind == FUPR_OP_CONV) {
    s.R = d.conv.R; s.S = d.conv.S; s.stride = d.conv.stride;
    const double crs = (double)d.conv.C * d.conv.R * d.conv.S;
    s.flops = 2.0 * crs * d.conv.K * (double)s.M;
    double res_b = 0.0;
    if (d.res >= 0) res_b = es * (double)s.M * m->tensors[d.res].C;
    s.bytes = in_b + out_b + res_b + es * crs * d.conv.K + 4.0 * d.conv.K;
    if (d.epilogue & FUPR_FUSE_CAT) {
      // the second tensor's pixels that are read (one per output pixel); the zero
      // channels between the two tensors are neither read nor multiplied
      const double c2 = (double)m->tensors[d.in2].C;
      s.bytes += es * (double)s.M * c2 - es * ((double)d.conv.C - ti.C - c2) * d.conv.K;
      s.flops = 2.0 * (ti.C + c2) * d.conv.K * (double)s.M;
      s.C = ti.C + (int)c2;
    }
    const bool scatter = (d.epilogue & FUPR_FUSE_SCATTER) != 0;
    if (scatter)   // conv.K channels of the updated tensor read and written, and the index list
      s.bytes = in_b + 2.0 * es * (double)s.M * d.conv.K + es * crs * d.conv.K + 8.0 * d.conv.K;
    if (scatter) s.K = d.conv.K;
    s.kernel = conv_kernel_name(d.conv, m->dt, batch, ti.H, ti.W, scatter,
                                (d.epilogue & FUPR_FUSE_CAT) != 0);
  } else {
    s.R = s.S = d.kind == FUPR_OP_MAXPOOL ? d.conv.R : ti.H;
    s.stride = d.kind == FUPR_OP_MAXPOOL ? d.conv.stride : 1;
    s.flops = 0.0;
    s.bytes = in_b + out_b;
    s.kernel = d.kind == FUPR_OP_MAXPOOL ? "maxpool" : "global_avgpool";
  }
  *out = s;
  return FUPR_OK;
}

namespace {
// The one-kernel schedule will run (given tensors of the planned strides).
bool one_kernel(const fupr_model* m) {
  return m->resident_ok && m->res_dev && m->schedule == FUPR_SCHEDULE_AUTO;
}
}  // namespace

extern "C" int32_t fupr_model_num_launches(const fupr_model* m) {
  if (!m) return 0;
  return one_kernel(m) ? 1 : (int32_t)launches_of(m).size();
}

extern "C" fupr_status fupr_model_launch_stats(const fupr_model* m, int32_t batch, int32_t launch,
                                               fupr_op_stats* out) {
  if (!m || !out) return FUPR_ERR_NULL;
  if (batch <= 0 || launch < 0 || launch >= fupr_model_num_launches(m)) return FUPR_ERR_ARG;
  if (!one_kernel(m)) {
    const Launch l = launches_of(m)[launch];
    fupr_status st = fupr_model_op_stats(m, batch, l.first, out);
    if (st != FUPR_OK || l.count == 1) return st;
    out->n_ops = l.count;
    if (m->ops[l.first + 1].kind == FUPR_OP_CONV) {
      // two convolutions in one kernel: both outputs are written, the first one's
      // is not read back
      fupr_op_stats second;
      st = fupr_model_op_stats(m, batch, l.first + 1, &second);
      if (st != FUPR_OK) return st;
      const TensorInfo& mid = m->tensors[l.first + 1];
      out->flops += second.flops;
      out->bytes += second.bytes - (double)elem_size(m->dt) * batch * (double)mid.H * mid.W * mid.C;
      out->kernel = "conv1x1s_256f+conv1x1";
      return FUPR_OK;
    }
    // convolution + pool in one kernel: the convolution's flops; its input and
    // parameters read, the pool's output written
    fupr_op_stats pool;
    st = fupr_model_op_stats(m, batch, l.first + 1, &pool);
    if (st != FUPR_OK) return st;
    const double es = (double)elem_size(m->dt);
    const TensorInfo& mid = m->tensors[l.first + 1];
    const double mid_b = es * batch * (double)mid.H * mid.W * mid.C;
    out->bytes += pool.bytes - 2.0 * mid_b;
    out->kernel = "stem7x7_maxpool";
    return FUPR_OK;
  }
  // one kernel: all flops; the image in, the result out, every parameter once
  const double es = (double)elem_size(m->dt);
  const TensorInfo& t0 = m->tensors.front();
  const TensorInfo& tl = m->tensors.back();
  fupr_op_stats s{};
  s.first_op = 0;
  s.n_ops = (int32_t)m->ops.size();
  s.M = batch;
  s.C = t0.C;
  s.K = tl.C;
  s.R = t0.H;
  s.S = t0.W;
  s.stride = 1;
  s.bytes = es * batch * ((double)t0.C * t0.H * t0.W + (double)tl.C * tl.H * tl.W);
  for (size_t i = 0; i < m->ops.size(); ++i) {
    fupr_op_stats o;
    const fupr_status st = fupr_model_op_stats(m, batch, (int32_t)i, &o);
    if (st != FUPR_OK) return st;
    s.flops += o.flops;
    const fupr_op_desc& d = m->ops[i];
    if (d.kind == FUPR_OP_CONV)
      s.bytes += es * (double)d.conv.C * d.conv.R * d.conv.S * d.conv.K + 4.0 * d.conv.K;
  }
  s.kernel = "resident_network";
  *out = s;
  return FUPR_OK;
}

extern "C" fupr_status fupr_graph_create(const fupr_model* m, const fupr_tensor* input,
                                         const fupr_tensor* output, void* workspace,
                                         size_t workspace_bytes, void* stream, fupr_graph** out) {
  if (!out) return FUPR_ERR_NULL;
  if (!stream) return FUPR_ERR_ARG;
  hipStream_t hs = reinterpret_cast<hipStream_t>(stream);
  fupr_graph* g = new (std::nothrow) fupr_graph;
  if (!g) return FUPR_ERR_ARG;
  if (hipStreamBeginCapture(hs, hipStreamCaptureModeThreadLocal) != hipSuccess) {
    delete g;
    return FUPR_ERR_LAUNCH;
  }
  const fupr_status st = run(m, input, output, workspace, workspace_bytes, stream, nullptr);
  const hipError_t e = hipStreamEndCapture(hs, &g->graph);
  if (st != FUPR_OK || e != hipSuccess || !g->graph) {
    if (g->graph) (void)hipGraphDestroy(g->graph);
    delete g;
    return st != FUPR_OK ? st : FUPR_ERR_LAUNCH;
  }
  if (hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0) != hipSuccess) {
    (void)hipGraphDestroy(g->graph);
    delete g;
    return FUPR_ERR_LAUNCH;
  }
  *out = g;
  return FUPR_OK;
}

extern "C" fupr_status fupr_graph_launch(const fupr_graph* g, void* stream) {
  if (!g || !g->exec) return FUPR_ERR_NULL;
  return hipGraphLaunch(g->exec, reinterpret_cast<hipStream_t>(stream)) == hipSuccess
             ? FUPR_OK
             : FUPR_ERR_LAUNCH;
}

extern "C" void fupr_graph_destroy(fupr_graph* g) {
  if (!g) return;
  if (g->exec) (void)hipGraphExecDestroy(g->exec);
  if (g->graph) (void)hipGraphDestroy(g->graph);
  delete g;
}
