// C ABI of the library (include/morello_mi355x.h) and the host side of the
// solver: descriptor validation, coordinate system (Section 4.1), dependency
// levels of the bottom-up fill (Section 4 run in reverse), launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <condition_variable>
#include <cstring>
#include <functional>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/morello_mi355x.h"
#include "compress.h"
#include "dev_params.h"

using namespace mrl;

static thread_local char g_err[512] = "";

static int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                              \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return fail(MRL_E_HIP, "%s: %s", #expr, hipGetErrorString(e_));          \
  } while (0)

struct mrl_target {
  mrl_target_desc d;
};

namespace {

constexpr size_t kAlign = 256;
constexpr uint32_t kQueryChunk = 4096;
#ifndef MRL_SECOND_ON_CELLS
#define MRL_SECOND_ON_CELLS 1
#endif
constexpr bool kSecondOnCells = MRL_SECOND_ON_CELLS;
constexpr uint32_t kLookupChunk = 65536;   // points per launch of a lookup in the box lists
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Host-side compiled lattice: everything derived from (target, lattice).
struct Compiled {
  DevParams P;
  std::vector<TileEntry> tiles;
  std::vector<uint32_t> level_shapes;     // shapes grouped by dependency level, ascending inside a level
  std::vector<uint32_t> level_off;        // [n_levels + 1]
  std::vector<uint32_t> sizes[4];
  Geo geo;
  uint32_t merge_order[16];
  uint32_t n_shapes;
  uint64_t n_specs;
  std::vector<uint8_t> mk_entry;          // [256][V]
  uint32_t max_task;                      // entries of one unit = ncombo * V
  int lay_axis[5], dt_axis[5];            // coordinate axis of the operand's bit, -1 if none
  mrl_target_desc target;
  mrl_lattice_desc lat;                   // sizes pointers re-pointed to this->sizes
  // Pinned image of the uploaded head of the scratch buffer (counters .. mk_entry), built at the
  // first solve and patched per call (device pointers).
  mutable char* staging = nullptr;
  mutable std::mutex solve_mu;            // solves of one compiled lattice take turns (they share the image)
  ~Compiled() { if (staging) (void)hipHostFree(staging); }
};

// Offsets of the fixed part of the scratch buffer.
struct FixedLayout {
  size_t counters, params, tiles, level_shapes, shape_class, level_off, mk_entry, list_whole, list_slice, list_wide, list_cnt, fitmap, maskD, maskC, mask2D, mask2C, colD, colC, lineD, lineC, prefD, prefC, tile_tmp, tile_tmp2, totals,
      q_idx, q_cost, q_arg, upload_end, end;
  uint32_t n_words;
};

// Whether the pass on the second merge axis a1 runs on the cells, before the boxes are made: the
// first axis a0 and a1 have strides of whole mask words, a1 lies outside a0 and has at most 64 steps.
bool second_on_cells(const Compiled& c, uint32_t* a0_out, uint32_t* a1_out) {
  const Geo& g = c.geo;
  uint32_t a0 = 0, a1 = 0, found = 0;
  for (uint32_t q = 0; q < g.ndim && found < 2; q++) {
    const uint32_t a = c.merge_order[q];
    if (g.ext[a] <= 1) continue;
    if (found++ == 0) a0 = a; else a1 = a;
  }
  if (a0_out) *a0_out = a0;
  if (a1_out) *a1_out = a1;
  return kSecondOnCells && found == 2 && g.stride[a0] % 64 == 0 && g.stride[a1] % (g.stride[a0] * g.ext[a0]) == 0 && g.ext[a1] <= 64;
}

FixedLayout fixed_layout(const Compiled& c) {
  FixedLayout f;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  f.n_words = (uint32_t)((c.n_specs + 63) / 64);
  // uploaded in one copy: counters (zero), parameters, tile lists, level lists, microkernel table
  f.counters = take(sizeof(Counters));
  f.params = take(sizeof(DevParams));
  f.tiles = take(c.tiles.size() * sizeof(TileEntry) + 8);
  f.level_shapes = take(c.level_shapes.size() * 4);
  f.level_off = take(c.level_off.size() * 4);
  f.mk_entry = take(c.mk_entry.size());
  f.upload_end = o;
  f.shape_class = take(c.level_shapes.size() * 4);
  f.list_whole = take((size_t)c.n_shapes * 4);
  f.list_slice = take((size_t)c.n_shapes * c.P.npass * 4);
  f.list_wide = take((size_t)c.n_shapes * c.P.npass * 4);
  f.list_cnt = take(4 * c.level_off.size() * 4);
  f.fitmap = take((size_t)f.n_words * 8 + 16);
  f.maskD = take((size_t)f.n_words * 8);
  f.maskC = take((size_t)f.n_words * 8);
  f.mask2D = f.mask2C = f.colD = f.colC = 0;
  if (second_on_cells(c, nullptr, nullptr)) {
    uint32_t a1 = 0;
    second_on_cells(c, nullptr, &a1);
    f.mask2D = take((size_t)f.n_words * 8);
    f.mask2C = take((size_t)f.n_words * 8);
    f.colD = take((size_t)(c.n_specs / c.geo.ext[a1]) * 8);
    f.colC = take((size_t)(c.n_specs / c.geo.ext[a1]) * 8);
  }
  {
    // line-major copies of the two masks: one bit per cell, 64-bit words per line of the first merge axis
    uint32_t e0 = c.geo.ext[c.merge_order[0]];
    for (uint32_t q = 0; q < c.geo.ndim; q++) if (c.geo.ext[c.merge_order[q]] > 1) { e0 = c.geo.ext[c.merge_order[q]]; break; }
    const size_t line_bytes = (size_t)(c.n_specs / e0) * ((e0 + 63) / 64) * 8;
    f.lineD = take(line_bytes);
    f.lineC = take(line_bytes);
  }
  f.prefD = take((size_t)f.n_words * 4);
  f.prefC = take((size_t)f.n_words * 4);
  f.tile_tmp = take((c.n_specs / kScanTileItems + 2) * 4);
  f.tile_tmp2 = take((c.n_specs / kScanTileItems + 2) * 4);
  f.totals = take(64);
  f.q_idx = take(kQueryChunk * 8);
  f.q_cost = take(kQueryChunk * 8);
  f.q_arg = take(kQueryChunk * 2);
  f.end = o;
  return f;
}

// per box while merging: bcell, blen, alive, next, pos, and for the dense copies of the live boxes
// cell2, len2, alive2, pos2; a flag per 256 boxes.  Per final box: fcell, flen, fv0, fv1
size_t work_bytes(uint64_t nb) { return 5 * align_up(nb * 4) + 2 * align_up(nb * 16) + 2 * align_up(nb) + align_up((nb / 256 + 1) * 4); }
size_t final_bytes(uint64_t nb) { return align_up(nb * 4) + align_up(nb * 16) + 2 * align_up(nb * 8); }

uint32_t ipow(uint32_t b, uint32_t e) { uint32_t r = 1; while (e--) r *= b; return r; }

int32_t validate_target(const mrl_target_desc* d) {
  if (!d) return fail(MRL_E_INVAL, "target descriptor is NULL");
  if (d->n_levels < 1 || d->n_levels > MRL_MAX_LEVELS) return fail(MRL_E_INVAL, "n_levels must be 1..4");
  if (d->n_microkernels > MRL_MAX_MK) return fail(MRL_E_INVAL, "too many microkernels");
  for (uint32_t j = 0; j < d->n_microkernels; j++) {
    if (d->mk[j].kind > MRL_MK_VEC_RELU) return fail(MRL_E_INVAL, "unknown microkernel kind %u", d->mk[j].kind);
    if (d->mk[j].lanes < 1) return fail(MRL_E_INVAL, "microkernel lanes must be >= 1");
    if (d->mk[j].kind != MRL_MK_SCALAR_FMA && d->mk[j].kind != MRL_MK_SCALAR_ADDRELU && d->mk[j].kind != MRL_MK_SCALAR_MOVE &&
        d->mk[j].kind != MRL_MK_SCALAR_ADD && d->mk[j].kind != MRL_MK_SCALAR_RELU && d->n_levels < 2)
      return fail(MRL_E_INVAL, "vector microkernels need a level 1");
  }
  return MRL_OK;
}

int32_t compile(const mrl_target_desc& T, const mrl_lattice_desc* L, Compiled& c) {
  if (!L) return fail(MRL_E_INVAL, "lattice descriptor is NULL");
  if (L->kind > MRL_KIND_BIAS_ADD_RELU_SPLIT) return fail(MRL_E_INVAL, "unknown spec kind %u", L->kind);
  // A parallel lattice is a Matmul lattice (same operator, operands and coordinates) with more
  // rewrites; a bounded one is the lattice of its operator with more coordinates; a Matmul whose
  // Moves are Move Specs is a Matmul lattice with other Move costs; the composition of two Matmuls
  // has the fused Spec's structure (four operands and an intermediate between two stages).
  const bool chain = L->kind == MRL_KIND_MATMUL_CHAIN;
  // The bias add alone has the operands and coordinates of the bias-add + ReLU (other microkernels
  // apply to it); the ReLU alone has two tensors; the bias-add + ReLU with its own bufferize has
  // more rewrites.
  const bool add_only = L->kind == MRL_KIND_BIAS_ADD, relu_only = L->kind == MRL_KIND_RELU, split = L->kind == MRL_KIND_BIAS_ADD_RELU_SPLIT;
  const bool parallel = L->kind == MRL_KIND_MATMUL_PARALLEL, move_specs = L->kind == MRL_KIND_MOVE, moves = L->kind == MRL_KIND_MATMUL_MOVES;
  const bool bounded = L->kind >= MRL_KIND_MATMUL_BOUNDED && L->kind <= MRL_KIND_FUSED_BOUNDED;
  const uint32_t kind = parallel || moves ? (uint32_t)kKindM : bounded ? L->kind - MRL_KIND_MATMUL_BOUNDED : move_specs ? (uint32_t)kKindV
                        : chain ? (uint32_t)kKindF : add_only || split ? (uint32_t)kKindE : relu_only ? (uint32_t)kKindR : L->kind;
  if (parallel && T.threads < 1) return fail(MRL_E_INVAL, "a MATMUL_PARALLEL lattice needs threads >= 1");
  if ((move_specs || moves) && T.line_bytes < 1) return fail(MRL_E_INVAL, "MOVE and MATMUL_MOVES lattices need line_bytes >= 1");
  c.target = T;
  c.lat = *L;
  DevParams& P = c.P;
  memset(&P, 0, sizeof P);
  P.kind = kind;
  P.par = parallel ? 1u : 0u;
  P.threads = parallel ? T.threads : 1u;
  P.sync = T.sync_cost;
  // memory bounds: one axis per level of finite capacity, values 0, 1, 2, 4, ... up to the capacity
  P.bounded = bounded ? 1u : 0u;
  P.Q = 1;
  for (uint32_t l = 0; l < 4; l++) P.lim_of_level[l] = kNoBit;
  if (bounded) {
    for (uint32_t l = 0; l < T.n_levels; l++) {
      if (T.capacity_bytes[l] == UINT64_MAX) continue;
      uint32_t nq = 1;
      while (nq < 64 && (1ull << (nq - 1)) <= T.capacity_bytes[l]) nq++;
      P.lim_of_level[l] = P.nlim;
      P.lim_nq[P.nlim++] = nq;
    }
  }
  bool packed = false;       // some tensor may be packed in strips
  for (uint32_t i = 0; i < 5; i++) {
    if (L->layout_coord[i] > 2) return fail(MRL_E_INVAL, "layout_coord[%u] must be 0, 1 or 2", i);
    if (L->layout_coord[i] == 2) {
      if (!(move_specs || moves)) return fail(MRL_E_INVAL, "packed layouts (layout_coord 2) only in MOVE and MATMUL_MOVES lattices");
      if (T.strip < 2 || T.strip % 2) return fail(MRL_E_INVAL, "packed layouts need an even strip >= 2");
      packed = true;
    }
  }
  P.strip = T.strip;
  P.xw = packed ? 4u : 2u;
  if (move_specs) {
    // contiguousness (a packed tensor has three physical dimensions) and aligned flag of the source, then of the destination
    P.nlim = 4;
    P.lim_nq[0] = packed ? 4 : 3; P.lim_nq[1] = 2; P.lim_nq[2] = packed ? 4 : 3; P.lim_nq[3] = 2;
  }
  for (uint32_t a = P.nlim; a-- > 0;) { P.lim_stride[a] = P.Q; P.Q *= P.lim_nq[a]; }
  P.gather = bounded || move_specs || moves ? 1u : 0u;
  P.moves = moves ? 1u : 0u;
  P.chain = chain ? 1u : 0u;
  P.split = split ? 1u : 0u;
  P.line_bytes = T.line_bytes;
  P.line_mask = T.line_bytes && (T.line_bytes & (T.line_bytes - 1)) == 0 ? T.line_bytes - 1 : 0;
  for (int l = 0; l < 4; l++) P.weight[l] = T.level_weight[l];
  P.nops = kind == kKindF ? 4 : kind == kKindV || kind == kKindR ? 2 : 3;
  P.nlv = kind == kKindF ? 5 : kind == kKindV || kind == kKindR ? 2 : 3;
  P.NL = T.n_levels;
  P.npass = kind == kKindF ? P.NL : 1;
  P.ncombo = ipow(P.NL, P.nops);
  uint64_t max_vol = 1;
  uint32_t maxs = 0;
  for (int d = 0; d < 4; d++) {
    uint32_t n = L->n_sizes[d];
    if (n < 1 || n > MRL_MAX_SIZES || !L->sizes[d]) return fail(MRL_E_INVAL, "n_sizes[%d] must be 1..%d", d, MRL_MAX_SIZES);
    c.sizes[d].assign(L->sizes[d], L->sizes[d] + n);
    // (no rewrite of a fused Spec changes k: a fused lattice may cover any stretch of k values)
    if (c.sizes[d][0] != 1 && !(d == 2 && kind == kKindF && !chain)) return fail(MRL_E_INVAL, "sizes[%d] must start with 1", d);
    for (uint32_t j = 1; j < n; j++)
      if (c.sizes[d][j] <= c.sizes[d][j - 1]) return fail(MRL_E_INVAL, "sizes[%d] must be strictly ascending", d);
    c.lat.sizes[d] = c.sizes[d].data();
    P.nsz[d] = n;
    for (uint32_t j = 0; j < n; j++) P.sizes[d][j] = c.sizes[d][j];
    max_vol *= c.sizes[d][n - 1];
    if (max_vol >= (1ull << 48)) return fail(MRL_E_INVAL, "b*m*k*n must stay below 2^48");
    maxs = std::max(maxs, n);
  }
  if (kind != kKindM && !chain && L->n_sizes[0] != 1) return fail(MRL_E_INVAL, "this kind has no batch dimension");
  if ((kind == kKindE || kind == kKindR) && L->n_sizes[2] != 1) return fail(MRL_E_INVAL, "BIAS_ADD_RELU, BIAS_ADD and RELU have no k dimension");
  if (kind == kKindV && L->n_sizes[2] != 1) return fail(MRL_E_INVAL, "MOVE has no k dimension");
  if (moves && L->n_sizes[0] != 1) return fail(MRL_E_INVAL, "MATMUL_MOVES has no batch dimension");
  P.shape_stride[3] = 1;
  for (int d = 2; d >= 0; d--) P.shape_stride[d] = P.shape_stride[d + 1] * P.nsz[d + 1];
  c.n_shapes = P.shape_stride[0] * P.nsz[0];

  // variant bits: layout bits (operand order) above dtype bits (operand order)
  for (int i = 0; i < 5; i++) { P.lay_bit[i] = P.dt_bit[i] = kNoBit; c.lay_axis[i] = c.dt_axis[i] = -1; }
  for (uint32_t i = 0; i < P.nops; i++) {
    P.nlay += L->layout_coord[i];          // bits of the layout field
    P.lay_w[i] = L->layout_coord[i];
    P.ndt += L->dtype_coord[i] ? 1 : 0;
    if (L->dtype_coord[i] && !(kind == kKindV || (kind == kKindM && i < 2))) return fail(MRL_E_INVAL, "dtype bit only on MatmulAccum inputs and on the tensors of a MOVE");
    if (L->base_dtype_bytes[i] != 4 && !(L->base_dtype_bytes[i] == 2 && (kind == kKindM || kind == kKindV)))
      return fail(MRL_E_INVAL, "base_dtype_bytes[%u] must be 4 (or 2 on a MatmulAccum or a MOVE)", i);
    P.base_bf16[i] = L->base_dtype_bytes[i] == 2;
    // (the second Matmul of a composition accumulates into out, as every Matmul does)
    P.access[i] = kind == kKindM ? (i == 2 ? kRmw : kRead) : (i == P.nops - 1 ? (chain ? kRmw : kWrite) : kRead);
    P.lvpow[i] = ipow(P.NL, P.nops - 1 - i);
    P.pack_shift[i] = 2 * (P.nops - 1 - i);
  }
  P.V = 1u << (P.nlay + P.ndt);
  P.log2V = P.nlay + P.ndt;

  if (P.V > (P.gather ? 64u : 16u)) return fail(MRL_E_INVAL, "too many layout/dtype bits");
  {
    uint32_t axis = 4 + P.nlv + P.nlim, seen_l = 0, seen_d = 0;
    for (uint32_t i = 0; i < P.nops; i++)
      if (L->layout_coord[i]) { seen_l += L->layout_coord[i]; c.lay_axis[i] = (int)axis++; P.lay_bit[i] = P.ndt + P.nlay - seen_l; }
    for (uint32_t i = 0; i < P.nops; i++)
      if (L->dtype_coord[i]) { c.dt_axis[i] = (int)axis++; P.dt_bit[i] = P.ndt - 1 - seen_d++; }
  }
  if ((uint64_t)P.ncombo * P.npass * P.V * P.Q >= (1ull << 32)) return fail(MRL_E_INVAL, "too many entries per shape");
  P.G = P.ncombo * P.npass * P.V * P.Q;
  c.n_specs = (uint64_t)c.n_shapes * P.G;
  if (c.n_specs >= (1ull << 32)) return fail(MRL_E_INVAL, "lattice has %llu specs; the limit is 2^32-1", (unsigned long long)c.n_specs);

  // target
  for (int l = 0; l < 4; l++) {
    P.cap[l] = T.capacity_bytes[l];
    P.zero[l] = T.zero_coef[l];
  }
  P.convert = T.convert_coef;
  P.s = T.loop_overhead;
  P.nmk = T.n_microkernels;
  for (uint32_t j = 0; j < P.nmk; j++) { P.mk_kind[j] = T.mk[j].kind; P.mk_lanes[j] = T.mk[j].lanes; P.mk_cost[j] = T.mk[j].cost; }

  // rewrite ids
  P.maxs = maxs;
  P.move_base = P.nmk;
  P.tile_base = P.move_base + P.nops * (P.NL - 1) * 2 * P.xw;
  P.buf_id = P.tile_base + 4 * maxs;
  P.par_base = P.buf_id + 1;
  if ((parallel ? P.par_base + 4 * maxs : P.buf_id + P.NL) >= kNone) return fail(MRL_E_INVAL, "rewrite ids do not fit 16 bits");

  // Moves: coefficient per (operand, src, dst, transposed) and the list of Moves that can occur
  for (uint32_t i = 0; i < (move_specs || moves ? 0u : P.nops); i++)
    for (uint32_t src = 0; src < P.NL; src++)
      for (uint32_t dst = 0; dst < src; dst++)
        for (uint32_t x = 0; x < 2; x++) {
          if (x && !L->layout_coord[i]) continue;
          const uint32_t ld = T.load_coef[src][dst][x], st = T.store_coef[dst][src][x];
          uint64_t cf = 0;
          if (P.access[i] != kWrite) { if (!ld) continue; cf += ld; }
          if (P.access[i] != kRead) { if (!st) continue; cf += st; }
          if (cf > UINT32_MAX) return fail(MRL_E_INVAL, "Move coefficients too large");
          P.mcoef[i][src][dst][x] = (uint32_t)cf;
        }
  for (uint32_t i = 0; i < P.nops; i++) P.can_convert[i] = L->dtype_coord[i] && P.access[i] == kRead;

  // microkernels: the level / layout / dtype part of each predicate, per (pack, variant)
  c.mk_entry.assign((size_t)256 * P.V, 0);
  for (uint32_t pack = 0; pack < 256; pack++)
    for (uint32_t v = 0; v < P.V; v++) {
      uint32_t lv[4], ly[4], bf[4];
      bool in_range = true;
      for (uint32_t i = 0; i < 4; i++) {
        lv[i] = i < P.nops ? (pack >> P.pack_shift[i]) & 3u : 0u;
        in_range = in_range && lv[i] < P.NL;
        ly[i] = i < P.nops && P.lay_bit[i] != kNoBit ? (v >> P.lay_bit[i]) & ((1u << P.lay_w[i]) - 1u) : 0u;
        bf[i] = i < P.nops ? (P.dt_bit[i] != kNoBit ? (v >> P.dt_bit[i]) & 1u : P.base_bf16[i]) : 0u;
      }
      if (!in_range || (P.nops < 4 && (pack >> (2 * P.nops)))) continue;
      uint8_t bits = 0;
      for (uint32_t j = 0; j < P.nmk; j++) {
        bool ok = false;
        const bool all_f32 = !(bf[0] | bf[1] | bf[2]);
        switch (T.mk[j].kind) {
          case MRL_MK_SCALAR_FMA: ok = P.kind == kKindM && !(lv[0] | lv[1] | lv[2]) && all_f32; break;
          case MRL_MK_BCAST_VEC_MULADD: {
            // rhs, out row-major; one row in whole packed strips is the same sequence of values
            auto rowlike = [&](uint32_t y) { return y == 0 || (y == 2 && T.strip % T.mk[j].lanes == 0); };
            ok = P.kind == kKindM && lv[0] == 0 && lv[1] == 1 && lv[2] == 1 && all_f32 && rowlike(ly[1]) && rowlike(ly[2]);
            break;
          }
          case MRL_MK_BF16_DOT: ok = P.kind == kKindM && lv[0] == 1 && lv[1] == 1 && lv[2] == 0 && bf[0] && bf[1] && !bf[2] && (P.lay_bit[1] == kNoBit || ly[1] == 1); break;
          case MRL_MK_SCALAR_ADDRELU: ok = P.kind == kKindE && !add_only && !(lv[0] | lv[1] | lv[2]); break;
          case MRL_MK_VEC_ADDRELU: ok = P.kind == kKindE && !add_only && lv[0] == 1 && lv[1] == 1 && lv[2] == 1 && !ly[0] && !ly[2]; break;
          case MRL_MK_SCALAR_ADD: ok = add_only && !(lv[0] | lv[1] | lv[2]); break;
          case MRL_MK_VEC_ADD: ok = add_only && lv[0] == 1 && lv[1] == 1 && lv[2] == 1 && !ly[0] && !ly[2]; break;
          case MRL_MK_SCALAR_RELU: ok = relu_only && !(lv[0] | lv[1]); break;
          case MRL_MK_VEC_RELU: ok = relu_only && lv[0] == 1 && lv[1] == 1 && !ly[0] && !ly[1]; break;
          // (the contiguousness / alignment part of the move microkernels' predicates is tested in the kernel)
          case MRL_MK_SCALAR_MOVE: ok = P.kind == kKindV && !(!bf[0] && bf[1]); break;
          case MRL_MK_VECTOR_MOVE:
          case MRL_MK_VECTOR_MOVE_ALIGNED:
            // (rows of strips: whether the strips are whole vectors is tested in the kernel, with the shape)
            ok = P.kind == kKindV && ((lv[0] == 1 && lv[1] > 1) || (lv[1] == 1 && lv[0] > 1)) && ly[0] != 1 && ly[1] != 1 &&
                 (ly[0] == 3) == (ly[1] == 3) && bf[0] == bf[1];
            break;
        }
        bits |= (uint8_t)((ok ? 1u : 0u) << j);
      }
      c.mk_entry[(size_t)pack * P.V + v] = bits;
    }

  // tiles: for (dim, size index) the smaller allowed sizes dividing it
  for (int d = 0; d < 4; d++) {
    P.tile_dim_ok[d] = kind == kKindM || d == 1 || d == 3;
    for (uint32_t j = 0; j < P.nsz[d]; j++) {
      P.tile_off[d][j] = (uint32_t)c.tiles.size();
      if (P.tile_dim_ok[d])
        for (uint32_t jt = 0; jt < j; jt++)
          if (c.sizes[d][j] % c.sizes[d][jt] == 0) {
            c.tiles.push_back(TileEntry{jt, c.sizes[d][j] / c.sizes[d][jt]});
          }
    }
    for (uint32_t j = P.nsz[d]; j <= (uint32_t)kMaxSizes; j++) P.tile_off[d][j] = (uint32_t)c.tiles.size();
  }

  // operand-level combos by rank
  P.nranks = P.nops * (P.NL - 1) + 1;
  {
    std::vector<std::pair<uint32_t, uint32_t>> order;
    for (uint32_t combo = 0; combo < P.ncombo; combo++) {
      uint32_t r = 0, x = combo;
      for (uint32_t i = 0; i < P.nops; i++) { r += x % P.NL; x /= P.NL; }
      order.push_back({r, combo});
    }
    std::sort(order.begin(), order.end());
    uint32_t q = 0;
    for (uint32_t r = 0; r <= P.nranks; r++) {
      while (q < order.size() && order[q].first < r) q++;
      P.rank_off[r] = q;
    }
    for (uint32_t i = 0; i < order.size(); i++) {
      const uint32_t combo = order[i].second;
      uint32_t pack = 0;
      for (uint32_t op = 0; op < P.nops; op++) pack |= ((combo / P.lvpow[op]) % P.NL) << P.pack_shift[op];
      uint32_t info = pack;
      for (uint32_t op = 0; op < P.nops; op++) info |= 1u << (8 + 4 * ((combo / P.lvpow[op]) % P.NL) + op);
      P.pos_info[i] = info;
    }
    for (uint32_t r = 0; r < P.nranks; r++) P.pos_info[P.rank_off[r]] |= (r + 1) << 24;     // first position of rank r
  }

  // dependency level of a shape = sum over tiled dims of the longest divisor chain below its size
  std::vector<uint32_t> depth[4];
  uint32_t n_lev = 1;
  for (int d = 0; d < 4; d++) {
    depth[d].assign(P.nsz[d], 0);
    uint32_t mx = 0;
    if (P.tile_dim_ok[d])
      for (uint32_t j = 0; j < P.nsz[d]; j++) {
        for (uint32_t q = P.tile_off[d][j]; q < P.tile_off[d][j + 1]; q++)
          depth[d][j] = std::max(depth[d][j], depth[d][c.tiles[q].jt] + 1);
        mx = std::max(mx, depth[d][j]);
      }
    n_lev += mx;
  }
  std::vector<uint32_t> lev(c.n_shapes);
  c.level_off.assign(n_lev + 1, 0);
  for (uint32_t sh = 0; sh < c.n_shapes; sh++) {
    uint32_t r = sh, l = 0;
    for (int d = 0; d < 4; d++) { l += depth[d][r / P.shape_stride[d]]; r %= P.shape_stride[d]; }
    lev[sh] = l;
    c.level_off[l + 1]++;
  }
  for (uint32_t l = 0; l < n_lev; l++) c.level_off[l + 1] += c.level_off[l];
  c.level_shapes.resize(c.n_shapes);
  {
    std::vector<uint32_t> cur(c.level_off.begin(), c.level_off.end() - 1);
    for (uint32_t sh = 0; sh < c.n_shapes; sh++) c.level_shapes[cur[lev[sh]]++] = sh;
  }

  // coordinate geometry and merge order: the memory-bound axes, n, k, m, b, the level axes,
  // layout bits, dtype bits, each group from its last axis to its first
  Geo& g = c.geo;
  memset(&g, 0, sizeof g);
  uint32_t nd = 0;
  for (int d = 0; d < 4; d++) g.ext[nd++] = P.nsz[d];
  for (uint32_t i = 0; i < P.nlv; i++) g.ext[nd++] = P.NL;
  for (uint32_t a = 0; a < P.nlim; a++) g.ext[nd++] = P.lim_nq[a];
  for (uint32_t i = 0; i < P.nops; i++) if (L->layout_coord[i]) g.ext[nd++] = 1u << L->layout_coord[i];
  for (uint32_t i = 0; i < P.ndt; i++) g.ext[nd++] = 2;
  if (nd > 16) return fail(MRL_E_INVAL, "more than 16 coordinate axes");
  g.ndim = nd;
  uint64_t s = 1;
  for (int a = (int)nd - 1; a >= 0; a--) { g.stride[a] = (uint32_t)s; s *= g.ext[a]; }
  g.n = (uint32_t)c.n_specs;
  {
    uint32_t q = 0;
    const int lim0 = 4 + (int)P.nlv, lay0 = lim0 + (int)P.nlim;
    for (int a = lay0 - 1; a >= lim0; a--) c.merge_order[q++] = (uint32_t)a;             // memory bounds
    for (int a = 3; a >= 0; a--) c.merge_order[q++] = (uint32_t)a;                       // n, k, m, b
    for (int a = lim0 - 1; a >= 4; a--) c.merge_order[q++] = (uint32_t)a;                // levels
    int n_lay_axes = 0;
    for (uint32_t i = 0; i < P.nops; i++) n_lay_axes += L->layout_coord[i] ? 1 : 0;
    for (int a = lay0 + n_lay_axes - 1; a >= lay0; a--) c.merge_order[q++] = (uint32_t)a;
    for (int a = (int)nd - 1; a >= lay0 + n_lay_axes; a--) c.merge_order[q++] = (uint32_t)a;
  }

  c.max_task = P.ncombo * P.V;
  if (c.max_task > 4096) return fail(MRL_E_INVAL, "too many entries per shape and intermediate level (%u > 4096)", c.max_task);
  return MRL_OK;
}


// compile() costs a few hundred microseconds for the larger lattices; repeated solves of the
// same (target, lattice) reuse the result.  Entries are immutable once published.
using CompiledPtr = std::shared_ptr<const Compiled>;

bool same_problem(const Compiled& c, const mrl_target_desc& T, const mrl_lattice_desc& L) {
  // (the whole target is compared, also the fields this lattice's kind does not use)
  if (memcmp(&c.target, &T, sizeof T) || c.lat.kind != L.kind) return false;
  if (memcmp(c.lat.layout_coord, L.layout_coord, sizeof L.layout_coord) ||
      memcmp(c.lat.dtype_coord, L.dtype_coord, sizeof L.dtype_coord) ||
      memcmp(c.lat.base_dtype_bytes, L.base_dtype_bytes, sizeof L.base_dtype_bytes)) return false;
  for (int d = 0; d < 4; d++) {
    if (L.n_sizes[d] != c.sizes[d].size() || !L.sizes[d]) return false;
    if (memcmp(L.sizes[d], c.sizes[d].data(), c.sizes[d].size() * sizeof(uint32_t))) return false;
  }
  return true;
}

int32_t get_compiled(const mrl_target_desc& T, const mrl_lattice_desc* L, CompiledPtr& out) {
  static std::mutex mu;
  static std::vector<CompiledPtr> cache;          // most recent last, at most 8
  if (L && L->kind <= MRL_KIND_BIAS_ADD_RELU_SPLIT) {
    std::lock_guard<std::mutex> lock(mu);
    for (size_t i = cache.size(); i-- > 0;)
      if (same_problem(*cache[i], T, *L)) { out = cache[i]; return MRL_OK; }
  }
  auto c = std::make_shared<Compiled>();
  const int32_t rc = compile(T, L, *c);
  if (rc) return rc;
  std::lock_guard<std::mutex> lock(mu);
  if (cache.size() >= 8) cache.erase(cache.begin());
  cache.push_back(c);
  out = c;
  return MRL_OK;
}

// A second stream (default priority, non-blocking) for work that is independent of what runs on
// the caller's stream: the wide items of a dependency level beside its other items, and one of the
// two box lists beside the other; with it the events and the pinned counters a solve needs.
constexpr size_t kPinnedCounts = 16 + 4 * 1024;   // u32: 16 for the box lists, then the level lists' lengths (4 per level)
struct Aux {
  hipStream_t stream = nullptr;
  std::vector<hipEvent_t> events;
  uint32_t* h_counts = nullptr;     // pinned: counts read back without stalling the other stream
  hipEvent_t timing[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};   // fill start, fill end, compression end and start, plan + pre-fill end, first dependency level
  int device = -1;
  bool busy = false;
};

// One set per solve in flight (solves on different host threads may overlap), kept for reuse.
struct AuxLease {
  Aux* a = nullptr;
  ~AuxLease();
};
std::mutex g_aux_mu;
std::vector<std::unique_ptr<Aux>> g_aux_pool;
AuxLease::~AuxLease() {
  if (a) { std::lock_guard<std::mutex> lock(g_aux_mu); a->busy = false; }
}

int32_t get_aux(size_t n_events, AuxLease& lease) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  Aux* aux = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_aux_mu);
    for (auto& p : g_aux_pool) if (!p->busy && p->device == dev) { aux = p.get(); break; }
    if (!aux) {
      g_aux_pool.emplace_back(new Aux);
      aux = g_aux_pool.back().get();
      aux->device = dev;
    }
    aux->busy = true;
  }
  lease.a = aux;
  if (!aux->stream) HIP_TRY(hipStreamCreateWithFlags(&aux->stream, hipStreamNonBlocking));
  if (!aux->h_counts) HIP_TRY(hipHostMalloc((void**)&aux->h_counts, kPinnedCounts * 4, hipHostMallocDefault));
  for (auto& e : aux->timing) if (!e) HIP_TRY(hipEventCreate(&e));
  while (aux->events.size() < n_events) {
    hipEvent_t e;
    HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    aux->events.push_back(e);
  }
  return MRL_OK;
}

}  // namespace

struct mrl_table {
  CompiledPtr cp;
  DevParams P;                // this table's copy: device pointers filled in by mrl_solve
  FixedLayout f;
  char* scratch;
  uint64_t* d_cost;
  uint16_t* d_arg;
  hipStream_t stream;
  const mrl_table* deps[2] = {nullptr, nullptr};      // a FUSED table: the tables it was solved against
  // final lists inside scratch: [0] decisions, [1] costs
  size_t list_off[2];
  uint64_t list_n[2];
  // Lookups in the box lists (mrl_query_compressed): bounding-box hierarchy per list and staging
  // for one chunk of points, allocated at the first such query and freed with the table.
  struct BoxIndex { IndexLevels L; BoxBounds* nodes = nullptr; };
  mutable BoxIndex index[2];
  mutable char* lookup_buf = nullptr;
  mutable std::mutex lookup_mu;
  mutable std::mutex query_mu;      // mrl_query stages through one area of the scratch buffer and the table's stream
  ~mrl_table() {
    for (auto& ix : index) if (ix.nodes) (void)hipFree(ix.nodes);
    if (lookup_buf) (void)hipFree(lookup_buf);
  }
};

// No exception leaves the library: host allocations (std::vector, std::make_shared, ...) can throw.
template <class F>
int32_t guarded(F&& body) noexcept {
  try { return body(); }
  catch (const std::bad_alloc&) { return fail(MRL_E_NOMEM, "host allocation failed"); }
  catch (const std::exception& e) { return fail(MRL_E_HIP, "internal error: %s", e.what()); }
  catch (...) { return fail(MRL_E_HIP, "internal error: unknown exception"); }
}

extern "C" {

const char* mrl_last_error(void) { return g_err; }

int32_t mrl_target_create(const mrl_target_desc* desc, mrl_target** out) {
  return guarded([&]() -> int32_t {
  if (!out) return fail(MRL_E_INVAL, "out is NULL");
  *out = nullptr;
  int32_t rc = validate_target(desc);
  if (rc) return rc;
  mrl_target* t = new (std::nothrow) mrl_target;
  if (!t) return fail(MRL_E_NOMEM, "host allocation failed");
  t->d = *desc;
  *out = t;
  return MRL_OK;
  });
}

void mrl_target_destroy(mrl_target* t) { delete t; }

int32_t mrl_geometry(const mrl_target* t, const mrl_lattice_desc* lat, uint32_t* n_dims, uint32_t* extents,
                     uint64_t* n_specs) {
  return guarded([&]() -> int32_t {
  if (!t) return fail(MRL_E_INVAL, "target is NULL");
  CompiledPtr cp;
  int32_t rc = get_compiled(t->d, lat, cp);
  if (rc) return rc;
  const Compiled& c = *cp;
  if (n_dims) *n_dims = c.geo.ndim;
  if (extents) for (uint32_t a = 0; a < c.geo.ndim; a++) extents[a] = c.geo.ext[a];
  if (n_specs) *n_specs = c.n_specs;
  return MRL_OK;
  });
}

int32_t mrl_table_bytes(const mrl_target* t, const mrl_lattice_desc* lat, size_t* cost_bytes, size_t* argmin_bytes,
                        size_t* scratch_bytes) {
  return guarded([&]() -> int32_t {
  if (!t) return fail(MRL_E_INVAL, "target is NULL");
  CompiledPtr cp;
  int32_t rc = get_compiled(t->d, lat, cp);
  if (rc) return rc;
  const Compiled& c = *cp;
  if (cost_bytes) *cost_bytes = c.n_specs * 8;
  if (argmin_bytes) *argmin_bytes = c.n_specs * 2;
  if (scratch_bytes) *scratch_bytes = fixed_layout(c).end + 2 * final_bytes(c.n_specs) + 2 * work_bytes(c.n_specs);
  return MRL_OK;
  });
}

}  // extern "C"

namespace {

// on_filled (optional) is called once, when the fill's last kernel is queued on the table's stream
// and before the compression starts: the dense table is then complete for any work ordered after
// that point of the stream.  It returns whether the caller now shares the table object; a shared
// one is not deleted when the rest of the solve fails (the sharer deletes it).
using FilledFn = std::function<bool(mrl_table*)>;

// late_deps (optional; then deps is NULL) hands over the tables a lattice reads only when the fill
// needs them: it is called once the work that reads no other table (work lists and the pre-fill)
// is queued, may wait on the host until those tables' fills are queued, and gives for each an
// event behind which the table is complete.  The pre-fill of a large table then runs beside the
// fill of the tables it will read, not after it.
using LateDepsFn = std::function<int32_t(const mrl_table* tables[2], hipEvent_t ready[2])>;

// Host threads that run the jobs of mrl_solve_graph.  They are kept between calls (a thread's
// first HIP calls are slow) and never end; every queued task gets a thread, since tasks wait for
// each other.  The pool is never destroyed: its threads may still wait in it when the process ends.
class Workers {
 public:
  void submit(std::function<void()> task) {
    std::lock_guard<std::mutex> lk(mu_);
    queue_.push_back(std::move(task));
    if (idle_ < queue_.size()) {
      try { std::thread([this] { loop(); }).detach(); }
      catch (...) { queue_.pop_back(); throw; }
    }
    cv_.notify_all();
  }

 private:
  void loop() {
    for (;;) {
      std::function<void()> task;
      {
        std::unique_lock<std::mutex> lk(mu_);
        idle_++;
        cv_.wait(lk, [&] { return !queue_.empty(); });
        idle_--;
        task = std::move(queue_.front());
        queue_.erase(queue_.begin());
      }
      task();
    }
  }
  std::mutex mu_;
  std::condition_variable cv_;
  std::vector<std::function<void()>> queue_;
  size_t idle_ = 0;
};
Workers& workers() { static Workers* w = new Workers; return *w; }

int32_t solve_impl(const mrl_target* t, const mrl_lattice_desc* lat, const mrl_table* const* deps, uint32_t n_deps,
                   void* d_cost, void* d_argmin, void* d_scratch, size_t scratch_bytes, void* hip_stream,
                   mrl_table** out, mrl_stats* stats, const FilledFn& on_filled, const LateDepsFn& late_deps = LateDepsFn()) {
  return guarded([&]() -> int32_t {
  if (!out) return fail(MRL_E_INVAL, "out is NULL");
  *out = nullptr;
  if (!t) return fail(MRL_E_INVAL, "target is NULL");
  if (!lat) return fail(MRL_E_INVAL, "lattice descriptor is NULL");
  if (!d_cost || !d_argmin || !d_scratch) return fail(MRL_E_INVAL, "device buffers must not be NULL");
  if (((uintptr_t)d_cost | (uintptr_t)d_argmin | (uintptr_t)d_scratch) % kAlign) return fail(MRL_E_INVAL, "device buffers must be 256-byte aligned");
  mrl_table* tab = new (std::nothrow) mrl_table;
  if (!tab) return fail(MRL_E_NOMEM, "host allocation failed");
  struct Guard { mrl_table* p; bool shared; ~Guard() { if (!shared) delete p; } } guard{tab, false};
  int32_t rc = get_compiled(t->d, lat, tab->cp);
  if (rc) return rc;
  const Compiled& c = *tab->cp;
  tab->P = c.P;
  DevParams& P = tab->P;

  const mrl_table* late_tables[2] = {nullptr, nullptr};
  hipEvent_t late_ready[2] = {nullptr, nullptr};
  // the tables this lattice reads: checked against it, their geometry and addresses into P
  auto bind_deps = [&]() -> int32_t {
    if (P.split) {
      if (n_deps != 2 || !deps || !deps[0] || !deps[1]) return fail(MRL_E_INVAL, "a BIAS_ADD_RELU_SPLIT lattice needs deps = {BIAS_ADD table, RELU table}");
      const Compiled& A = *deps[0]->cp;
      const Compiled& R = *deps[1]->cp;
      if (A.lat.kind != MRL_KIND_BIAS_ADD || R.lat.kind != MRL_KIND_RELU) return fail(MRL_E_INVAL, "deps must be {BIAS_ADD, RELU}");
      if (memcmp(&A.target, &t->d, sizeof t->d) || memcmp(&R.target, &t->d, sizeof t->d)) return fail(MRL_E_INVAL, "deps were solved for another target");
      if (A.sizes[1] != c.sizes[1] || A.sizes[3] != c.sizes[3] || R.sizes[1] != c.sizes[1] || R.sizes[3] != c.sizes[3])
        return fail(MRL_E_INVAL, "the deps must have this lattice's m and n size lists");
      if ((P.lay_bit[0] != kNoBit && A.P.lay_bit[0] == kNoBit) || (P.lay_bit[2] != kNoBit && R.P.lay_bit[1] == kNoBit))
        return fail(MRL_E_INVAL, "a tensor with a layout coordinate in the BIAS_ADD_RELU_SPLIT lattice needs one in the dep it is looked up in");
      P.costM = deps[0]->d_cost; P.costE = deps[1]->d_cost;
      tab->deps[0] = deps[0]; tab->deps[1] = deps[1];
      P.GM = A.P.G; P.VM = A.P.V; P.GE = R.P.G; P.VE = R.P.V;
      for (int i = 0; i < 3; i++) { P.layM[i] = A.P.lay_bit[i]; P.layE[i] = R.P.lay_bit[i]; }
    } else if (P.chain) {
      if (n_deps != 1 || !deps || !deps[0]) return fail(MRL_E_INVAL, "a MATMUL_CHAIN lattice needs deps = {MATMUL_ACCUM table}");
      const Compiled& M = *deps[0]->cp;
      if (M.P.kind != kKindM || M.P.par || M.P.bounded || M.P.moves) return fail(MRL_E_INVAL, "the dep must be a MATMUL_ACCUM table");
      if (memcmp(&M.target, &t->d, sizeof t->d)) return fail(MRL_E_INVAL, "the dep was solved for another target");
      if (M.sizes[0].size() != 1) return fail(MRL_E_INVAL, "MATMUL_ACCUM dep must have b pinned to 1");
      // both stages are looked up in it: (m, k, p) and (m, p, n)
      if (M.sizes[1] != c.sizes[1] || M.sizes[2] != c.sizes[2] || M.sizes[2] != c.sizes[0] || M.sizes[3] != c.sizes[0] || M.sizes[3] != c.sizes[3])
        return fail(MRL_E_INVAL, "the m list must equal the MATMUL_ACCUM dep's, and the p, k and n lists its k and n lists");
      if ((P.lay_bit[0] != kNoBit && M.P.lay_bit[0] == kNoBit) || (P.lay_bit[1] != kNoBit && M.P.lay_bit[1] == kNoBit) ||
          (P.lay_bit[2] != kNoBit && M.P.lay_bit[1] == kNoBit) || (P.lay_bit[3] != kNoBit && M.P.lay_bit[2] == kNoBit))
        return fail(MRL_E_INVAL, "a tensor with a layout coordinate in the MATMUL_CHAIN lattice needs one in the dep it is looked up in");
      if (M.P.ndt || M.P.base_bf16[0] || M.P.base_bf16[1] || M.P.base_bf16[2]) return fail(MRL_E_INVAL, "MATMUL_ACCUM dep must be f32");
      P.costM = deps[0]->d_cost;
      tab->deps[0] = deps[0];
      P.GM = M.P.G; P.VM = M.P.V; P.kM_first = 0; P.nkM = (uint32_t)M.sizes[2].size();
      for (int i = 0; i < 3; i++) P.layM[i] = M.P.lay_bit[i];
    } else if (P.kind == kKindF) {
      if (n_deps != 2 || !deps || !deps[0] || !deps[1]) return fail(MRL_E_INVAL, "a FUSED lattice needs deps = {MATMUL_ACCUM table, BIAS_ADD_RELU table}");
      const Compiled& M = *deps[0]->cp;
      const Compiled& E = *deps[1]->cp;
      if (M.P.kind != kKindM || M.P.par || E.P.kind != kKindE || E.lat.kind == MRL_KIND_BIAS_ADD)
        return fail(MRL_E_INVAL, "deps must be {MATMUL_ACCUM, BIAS_ADD_RELU (or BIAS_ADD_RELU_SPLIT)}");
      if (M.P.bounded != P.bounded || E.P.bounded != P.bounded) return fail(MRL_E_INVAL, "memory bounds on all three tables or on none");
      if ((P.lay_bit[0] != kNoBit && M.P.lay_bit[0] == kNoBit) || (P.lay_bit[1] != kNoBit && M.P.lay_bit[1] == kNoBit) ||
          (P.lay_bit[3] != kNoBit && E.P.lay_bit[2] == kNoBit))
        return fail(MRL_E_INVAL, "a tensor with a layout coordinate in the FUSED lattice needs one in the dep it is looked up in");
      if (memcmp(&M.target, &t->d, sizeof t->d) || memcmp(&E.target, &t->d, sizeof t->d)) return fail(MRL_E_INVAL, "deps were solved for another target");
      if (M.sizes[1] != c.sizes[1] || M.sizes[3] != c.sizes[3]) return fail(MRL_E_INVAL, "MATMUL_ACCUM dep has other size lists");
      {
        // the k list: the dep's, or a stretch of consecutive entries of it (a slab of the whole lattice)
        const auto at = std::find(M.sizes[2].begin(), M.sizes[2].end(), c.sizes[2][0]);
        if ((size_t)(M.sizes[2].end() - at) < c.sizes[2].size() || !std::equal(c.sizes[2].begin(), c.sizes[2].end(), at))
          return fail(MRL_E_INVAL, "the k list must be a stretch of the MATMUL_ACCUM dep's k list");
        P.kM_first = (uint32_t)(at - M.sizes[2].begin());
        P.nkM = (uint32_t)M.sizes[2].size();
      }
      if (M.sizes[0].size() != 1) return fail(MRL_E_INVAL, "MATMUL_ACCUM dep must have b pinned to 1");
      if (E.sizes[1] != c.sizes[1] || E.sizes[3] != c.sizes[3]) return fail(MRL_E_INVAL, "BIAS_ADD_RELU dep has other size lists");
      if (M.P.ndt || M.P.base_bf16[0] || M.P.base_bf16[1] || M.P.base_bf16[2]) return fail(MRL_E_INVAL, "MATMUL_ACCUM dep must be f32");
      P.costM = deps[0]->d_cost; P.costE = deps[1]->d_cost;
      tab->deps[0] = deps[0]; tab->deps[1] = deps[1];
      P.GM = M.P.G; P.VM = M.P.V; P.GE = E.P.G; P.VE = E.P.V; P.nszE_n = E.P.nsz[3];
      for (int i = 0; i < 3; i++) { P.layM[i] = M.P.lay_bit[i]; P.layE[i] = E.P.lay_bit[i]; }
    } else if (P.par) {
      if (n_deps != 1 || !deps || !deps[0]) return fail(MRL_E_INVAL, "a MATMUL_PARALLEL lattice needs deps = {MATMUL_ACCUM table of the same lattice}");
      const Compiled& M = *deps[0]->cp;
      if (M.P.kind != kKindM || M.P.par) return fail(MRL_E_INVAL, "the dep must be a MATMUL_ACCUM table");
      if (memcmp(&M.target, &t->d, sizeof t->d)) return fail(MRL_E_INVAL, "the dep was solved for another target");
      for (int d = 0; d < 4; d++) if (M.sizes[d] != c.sizes[d]) return fail(MRL_E_INVAL, "the MATMUL_ACCUM dep has other size lists");
      if (memcmp(M.lat.layout_coord, c.lat.layout_coord, sizeof c.lat.layout_coord) ||
          memcmp(M.lat.dtype_coord, c.lat.dtype_coord, sizeof c.lat.dtype_coord) ||
          memcmp(M.lat.base_dtype_bytes, c.lat.base_dtype_bytes, 3) || M.n_specs != c.n_specs || M.P.G != P.G)
        return fail(MRL_E_INVAL, "the MATMUL_ACCUM dep has other coordinates");
      P.costM = deps[0]->d_cost;
      tab->deps[0] = deps[0];
    } else if (P.moves) {
      if (n_deps != 1 || !deps || !deps[0]) return fail(MRL_E_INVAL, "a MATMUL_MOVES lattice needs deps = {MOVE table}");
      const Compiled& V = *deps[0]->cp;
      if (V.P.kind != kKindV) return fail(MRL_E_INVAL, "the dep must be a MOVE table");
      if (memcmp(&V.target, &t->d, sizeof t->d)) return fail(MRL_E_INVAL, "the dep was solved for another target");
      if (c.sizes[1] != V.sizes[1] || c.sizes[2] != V.sizes[1] || c.sizes[2] != V.sizes[3] || c.sizes[3] != V.sizes[3])
        return fail(MRL_E_INVAL, "the m, k and n size lists must all equal the MOVE table's row and column lists");
      bool any_lay = false, any_dt = false;
      for (int i = 0; i < 3; i++) { any_lay = any_lay || P.lay_bit[i] != kNoBit; any_dt = any_dt || P.dt_bit[i] != kNoBit || P.base_bf16[i]; }
      if (any_lay && (V.P.lay_bit[0] == kNoBit || V.P.lay_bit[1] == kNoBit)) return fail(MRL_E_INVAL, "the MOVE table needs layout bits on both tensors");
      if (P.xw == 4 && (V.P.lay_w[0] != 2 || V.P.lay_w[1] != 2)) return fail(MRL_E_INVAL, "the MOVE table needs the packed layouts on both tensors");
      if (any_dt && (V.P.dt_bit[0] == kNoBit || V.P.dt_bit[1] == kNoBit)) return fail(MRL_E_INVAL, "the MOVE table needs dtype bits on both tensors");
      if (V.P.dt_bit[0] == kNoBit && (V.P.base_bf16[0] || V.P.base_bf16[1])) return fail(MRL_E_INVAL, "a MOVE table without dtype bits must be f32");
      P.costM = deps[0]->d_cost;
      tab->deps[0] = deps[0];
      P.GV = V.P.G; P.VV = V.P.V; P.nszV = V.P.nsz[3]; P.QV = V.P.Q; P.qV_top = V.P.Q - 1;
      for (int a = 0; a < 4; a++) P.limV_stride[a] = V.P.lim_stride[a];
      for (int i = 0; i < 2; i++) { P.layV[i] = V.P.lay_bit[i]; P.dtV[i] = V.P.dt_bit[i]; }
    } else if (n_deps != 0) {
      return fail(MRL_E_INVAL, "only FUSED, MATMUL_PARALLEL, MATMUL_MOVES, MATMUL_CHAIN and BIAS_ADD_RELU_SPLIT lattices take deps");
    }
    return MRL_OK;
  };
  // (the lane-per-Spec kinds have no pre-fill to run ahead: they take their deps at once)
  const bool deps_late = (bool)late_deps && !P.gather && n_deps > 0;
  if (late_deps && !deps_late && n_deps > 0) {
    rc = late_deps(late_tables, late_ready);
    if (rc) return rc;
    deps = late_tables;
    for (uint32_t i = 0; i < n_deps; i++) HIP_TRY(hipStreamWaitEvent((hipStream_t)hip_stream, late_ready[i], 0));
  }
  if (!deps_late) { rc = bind_deps(); if (rc) return rc; }

  std::unique_lock<std::mutex> solve_lock(c.solve_mu);      // for the upload image, until the upload has run

  const FixedLayout f = fixed_layout(c);
  tab->f = f;
  if (scratch_bytes < f.end) return fail(MRL_E_NOMEM, "scratch buffer too small: %zu bytes given, at least %zu needed", scratch_bytes, f.end);
  char* base = (char*)d_scratch;
  hipStream_t st = (hipStream_t)hip_stream;
  tab->scratch = base; tab->d_cost = (uint64_t*)d_cost; tab->d_arg = (uint16_t*)d_argmin; tab->stream = st;

  Counters* d_ctr = (Counters*)(base + f.counters);
  DevParams* d_P = (DevParams*)(base + f.params);
  P.tiles = (const TileEntry*)(base + f.tiles);
  const uint32_t n_lev = (uint32_t)c.level_off.size() - 1;
  uint32_t* d_level_shapes = (uint32_t*)(base + f.level_shapes);
  uint32_t* d_shape_class = (uint32_t*)(base + f.shape_class);
  uint32_t* d_level_off = (uint32_t*)(base + f.level_off);
  uint32_t* d_list_whole = (uint32_t*)(base + f.list_whole);
  uint32_t* d_list_slice = (uint32_t*)(base + f.list_slice);
  uint32_t* d_list_wide = (uint32_t*)(base + f.list_wide);
  uint32_t* d_list_cnt = (uint32_t*)(base + f.list_cnt);
  uint32_t* d_fitmap = (uint32_t*)(base + f.fitmap);
  P.mk_entry = (const uint8_t*)(base + f.mk_entry);
  if (!c.staging) {
    HIP_TRY(hipHostMalloc((void**)&c.staging, f.upload_end, hipHostMallocDefault));
    memset(c.staging, 0, f.upload_end);
    if (!c.tiles.empty()) memcpy(c.staging + f.tiles, c.tiles.data(), c.tiles.size() * sizeof(TileEntry));
    memcpy(c.staging + f.level_shapes, c.level_shapes.data(), c.level_shapes.size() * 4);
    memcpy(c.staging + f.level_off, c.level_off.data(), c.level_off.size() * 4);
    memcpy(c.staging + f.mk_entry, c.mk_entry.data(), c.mk_entry.size());
  }
  memcpy(c.staging + f.params, &P, sizeof P);
  AuxLease lease;
  rc = get_aux(2 * (size_t)n_lev + 8, lease);
  if (rc) return rc;
  Aux* aux = lease.a;
  // Whichever way this function is left from here on, both streams have drained before the turn
  // for the upload image, the helper stream with its events and pinned counters, and (on
  // failure) the table object are given up: work queued on the streams may still use all of these.
  struct Drain {
    hipStream_t a, b;
    ~Drain() { (void)hipStreamSynchronize(a); (void)hipStreamSynchronize(b); }
  } drain{st, aux->stream};
  HIP_TRY(hipMemcpyAsync(base, c.staging, f.upload_end, hipMemcpyHostToDevice, st));

  // ---- fill: plan, then one launch (or two) per dependency level ----
  hipEvent_t* ev = aux->timing;
  size_t ev_used = 0;
  hipStream_t s2 = aux->stream;
  HIP_TRY(hipEventRecord(ev[0], st));
  bool prefill_timed = false, levels_timed = false;
  const hipEvent_t uploaded = aux->events[ev_used++];
  HIP_TRY(hipEventRecord(uploaded, st));
  if (P.gather) {
    // Memory bounds as coordinates (and Move Specs, and Matmuls whose Moves are Specs): every Spec is evaluated (no admissibility test, so every cell
    // counts as fitting for the compression); one launch per dependency level of shapes and rank
    // of level assignments, each over Specs that depend only on earlier launches.
    launch_fill_ones(d_fitmap, ((size_t)f.n_words + 2) * 8, st);
    const int gather_mode = P.kind == kKindV ? 1 : P.moves ? 2 : 0;
    for (uint32_t d = 0; d + 1 < n_lev + P.nranks; d++) {
      BoundSegs segs;
      segs.n = 0; segs.block0[0] = 0;
      auto flush = [&]() { launch_fill_bounded(d_P, gather_mode, d_level_shapes, segs, tab->d_cost, tab->d_arg, d_ctr, st); segs.n = 0; segs.block0[0] = 0; };
      for (uint32_t l = d < P.nranks ? 0 : d - (P.nranks - 1); l < n_lev && l <= d; l++) {
        const uint32_t r = d - l, ns = c.level_off[l + 1] - c.level_off[l];
        const uint64_t lanes = (uint64_t)ns * (P.rank_off[r + 1] - P.rank_off[r]) * P.npass * P.Q * P.V;
        const uint64_t blocks = (lanes + 255) / 256;
        if (!blocks) continue;
        if (segs.n == kBoundSegs || segs.block0[segs.n] + blocks >= (1ull << 31)) flush();
        if (blocks >= (1ull << 31)) return fail(MRL_E_INVAL, "a dependency level of the bounded lattice is too large for one launch");
        segs.first_shape[segs.n] = c.level_off[l]; segs.n_shapes[segs.n] = ns; segs.rank[segs.n] = r;
        segs.block0[segs.n + 1] = segs.block0[segs.n] + (uint32_t)blocks;
        segs.n++;
      }
      flush();
    }
  } else {
  // plan (with the pre-fill; a separate streaming kernel for tables it cannot serve), then the
  // host reads the list sizes back
  // A level assignment's fit bits (passive levels x variants) are whole 32-bit words of the map when
  // there are 32 or 64 of them: the plan kernel then stores them, and only the two pad words are zeroed.
  const bool fit_words = P.npass * P.V == 32 || P.npass * P.V == 64;
  if (fit_words) launch_zero_words((unsigned long long*)d_fitmap + f.n_words, 2, st);
  else launch_zero_words((unsigned long long*)d_fitmap, f.n_words + 2, st);
  // the plan kernel also streams (INF, NONE) over the tables when a shape's entries are whole 16-byte pieces
  // (not when the pre-fill runs beside the fill of the tables this lattice reads: see launch_fill_ones)
  const bool fused_prefill = P.G % 8 == 0 && !deps_late;
  launch_plan(d_P, c.n_shapes, P.npass, P.G, d_level_shapes, d_level_off, n_lev, d_shape_class, d_list_whole, d_list_slice,
              d_list_wide, d_list_cnt, d_fitmap, d_ctr, fused_prefill ? tab->d_cost : nullptr,
              fused_prefill ? tab->d_arg : nullptr, st);
  if (16 + 4 * (size_t)n_lev > kPinnedCounts) return fail(MRL_E_INVAL, "too many dependency levels (%u)", n_lev);
  const uint32_t* cnt = aux->h_counts + 16;            // pinned: the copy does not go through a staging buffer
  HIP_TRY(hipMemcpyAsync(aux->h_counts + 16, d_list_cnt, 4 * (size_t)n_lev * 4, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipEventRecord(aux->events[ev_used], st));
  hipEvent_t counts_ready = aux->events[ev_used++];
  if (!fused_prefill) {
    launch_fill_ones(tab->d_cost, c.n_specs * 8, st, deps_late);
    launch_fill_ones(tab->d_arg, c.n_specs * 2, st, deps_late);
  }
  HIP_TRY(hipEventRecord(ev[4], st));
  prefill_timed = true;
  HIP_TRY(hipEventSynchronize(counts_ready));
  if (deps_late) {
    // now the tables this lattice reads: their fills are queued (or the call waits here until
    // they are); the parameters go up once more, with their addresses, and the levels wait for them
    rc = late_deps(late_tables, late_ready);
    if (rc) return rc;
    deps = late_tables;
    rc = bind_deps();
    if (rc) return rc;
    memcpy(c.staging + f.params, &P, sizeof P);
    HIP_TRY(hipMemcpyAsync(d_P, c.staging + f.params, sizeof P, hipMemcpyHostToDevice, st));
    HIP_TRY(hipEventRecord(uploaded, st));
    for (uint32_t i = 0; i < n_deps; i++) HIP_TRY(hipStreamWaitEvent(st, late_ready[i], 0));
  }
  HIP_TRY(hipEventRecord(ev[5], st));
  levels_timed = true;
  bool wide_started = false;
  hipEvent_t wide_done = nullptr;          // recorded behind the last wide launch that the caller's stream has not waited for yet
  for (uint32_t l = 0; l < n_lev; l++) {
    const uint32_t first = c.level_off[l];
    const uint32_t n_small = cnt[l], n_slice = cnt[n_lev + l], n_wide = cnt[2 * n_lev + l], n_bigwhole = cnt[3 * n_lev + l];
    const uint32_t n_stretch = c.level_off[l + 1] - first;
    if (n_small + n_bigwhole > n_stretch || n_slice + n_wide > n_stretch * P.npass)
      return fail(MRL_E_HIP, "internal error: work lists of level %u overflow", l);
    // The wide items (slices with more tasks than an LDS slice of a wave holds) run on the helper
    // stream, level after level, without waiting for the other items: a tile of a wide slice
    // leads to the same slice of a smaller shape, in which at least as much fits, so that one is
    // wide as well, and wide items read nothing that the others write.  The others read entries
    // of any kind, so a level's launch on the caller's stream waits for the wide items of all
    // lower levels.  (With both kinds joined at every level the levels of the fused table took
    // 1.49 ms, the wide items setting the pace of most of them.)
    if (n_wide) {
      if (!wide_started) {
        HIP_TRY(hipEventRecord(aux->events[ev_used], st));
        HIP_TRY(hipStreamWaitEvent(s2, aux->events[ev_used++], 0));
        wide_started = true;
      }
      launch_fill_level(d_P, P.npass, P.G, c.max_task, d_list_whole + first, n_stretch, 0, 0,
                        d_list_slice + (size_t)first * P.npass, 0, d_list_wide + (size_t)first * P.npass, n_wide,
                        tab->d_cost, tab->d_arg, d_ctr, st, s2);
    }
    if (n_small + n_bigwhole + n_slice) {
      if (wide_done) { HIP_TRY(hipStreamWaitEvent(st, wide_done, 0)); wide_done = nullptr; }
      launch_fill_level(d_P, P.npass, P.G, c.max_task, d_list_whole + first, n_stretch, n_small, n_bigwhole,
                        d_list_slice + (size_t)first * P.npass, n_slice, d_list_wide + (size_t)first * P.npass, 0,
                        tab->d_cost, tab->d_arg, d_ctr, st, st);
    }
    if (n_wide) {
      // the next level's other items wait here
      HIP_TRY(hipEventRecord(aux->events[ev_used], s2));
      wide_done = aux->events[ev_used++];
    }
  }
  if (wide_done) HIP_TRY(hipStreamWaitEvent(st, wide_done, 0));
  }
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipEventRecord(ev[1], st));
  if (on_filled) {
    // on_filled may wait (host side) for other jobs, which may need this lattice's turn
    HIP_TRY(hipEventSynchronize(uploaded));
    solve_lock.unlock();
    guard.shared = on_filled(tab);
  }
  HIP_TRY(hipEventRecord(ev[3], st));

  // ---- compression ----
  const Geo& g = c.geo;
  uint32_t a0 = c.merge_order[0];
  for (uint32_t q = 0; q < g.ndim; q++) if (g.ext[c.merge_order[q]] > 1) { a0 = c.merge_order[q]; break; }
  unsigned long long* maskL[2] = {(unsigned long long*)(base + f.maskD), (unsigned long long*)(base + f.maskC)};
  uint32_t* prefL[2] = {(uint32_t*)(base + f.prefD), (uint32_t*)(base + f.prefC)};
  uint32_t* tile_tmp = (uint32_t*)(base + f.tile_tmp);
  uint32_t* d_tot = (uint32_t*)(base + f.totals);
  auto axis_sizes = [&](uint32_t a) -> const uint32_t* { return a < 4 ? (const uint32_t*)((char*)d_P + offsetof(DevParams, sizes) + a * sizeof(uint32_t) * kMaxSizes) : nullptr; };
  unsigned long long* lineL[2] = {(unsigned long long*)(base + f.lineD), (unsigned long long*)(base + f.lineC)};
  launch_head_flags(g, a0, tab->d_cost, tab->d_arg, d_fitmap, axis_sizes(a0), maskL[0], maskL[1], lineL[0], lineL[1], st);
  uint32_t a1 = 0;
  const bool on_cells = second_on_cells(c, nullptr, &a1);
  const unsigned long long* colL[2] = {nullptr, nullptr};
  if (on_cells) launch_zero_words((unsigned long long*)(base + f.colD), (uint32_t)((f.colC - f.colD) / 8 + c.n_specs / g.ext[a1]), st);
  // the two prefix sums side by side (each is three short kernels): the decisions' on the helper stream
  HIP_TRY(hipEventRecord(aux->events[ev_used], st));
  HIP_TRY(hipStreamWaitEvent(s2, aux->events[ev_used++], 0));
  if (on_cells) {
    // the pass on the second merge axis, on the cells: the box heads that remain go to a second mask
    unsigned long long* m2[2] = {(unsigned long long*)(base + f.mask2D), (unsigned long long*)(base + f.mask2C)};
    unsigned long long* cl[2] = {(unsigned long long*)(base + f.colD), (unsigned long long*)(base + f.colC)};
    launch_second_axis(g, a0, a1, false, maskL[0], lineL[0], d_fitmap, tab->d_cost, tab->d_arg, axis_sizes(a1), m2[0], cl[0], s2);
    launch_second_axis(g, a0, a1, true, maskL[1], lineL[1], d_fitmap, tab->d_cost, tab->d_arg, axis_sizes(a1), m2[1], cl[1], st);
    for (int w = 0; w < 2; w++) { maskL[w] = m2[w]; colL[w] = cl[w]; }
  }
  scan_mask_words(maskL[0], f.n_words, (uint32_t*)(base + f.tile_tmp2), prefL[0], d_tot + 0, s2);
  scan_mask_words(maskL[1], f.n_words, tile_tmp, prefL[1], d_tot + 1, st);
  HIP_TRY(hipEventRecord(aux->events[ev_used], s2));
  HIP_TRY(hipStreamWaitEvent(st, aux->events[ev_used++], 0));
  uint32_t h_tot[4] = {0, 0, 0, 0};
  HIP_TRY(hipMemcpyAsync(h_tot, d_tot, 8, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));

  // The two lists are merged side by side, the decisions on the helper stream: most of the
  // kernels are bound by latency, not bandwidth.  The host waits twice per list: for the number
  // of live boxes after the first pass (it sizes the grids of the later ones) and for the final
  // count (it places the final list); meanwhile the other list's stream has work queued.
  // Work areas at the end of the buffer, the final lists grow from the front.
  const uint64_t nbL[2] = {h_tot[0], h_tot[1]};
  const size_t wbL[2] = {work_bytes(nbL[0]), work_bytes(nbL[1])};
  size_t front = f.end;
  size_t needed = f.end + wbL[0] + wbL[1] + final_bytes(nbL[0]) + final_bytes(nbL[1]);   // upper bound until the final counts are known
  if (scratch_bytes < f.end + wbL[0] + wbL[1])
    return fail(MRL_E_NOMEM, "scratch buffer too small: %zu bytes given, up to %zu needed", scratch_bytes, needed);
  char* work_lo = base + (scratch_bytes - wbL[0] - wbL[1]) / kAlign * kAlign;
  if ((size_t)(work_lo - base) < f.end)
    return fail(MRL_E_NOMEM, "scratch buffer too small: %zu bytes given, up to %zu needed", scratch_bytes, needed);
  // per list: its arrays and the pass state.  Once the first pass has merged most boxes away, the
  // live ones move to dense arrays (cell2, len2, alive2) and get new indices 0..n-1, in order
  struct ListWork {
    uint32_t *bcell, *next, *pos, *cell2, *pos2, *block_linked, *d_cnt;
    char *blen, *len2;
    uint8_t *alive, *alive2;
    const uint8_t* old_alive = nullptr;     // set by the compaction, with remap
    const uint32_t* remap = nullptr;
    uint32_t n = 0, q_next = 0;
    uint8_t stamp = 0;
  } LW[2];
  hipStream_t stL[2] = {s2, st};
  uint32_t* tileL[2] = {(uint32_t*)(base + f.tile_tmp2), tile_tmp};
  // the passes in order; the trailing ones over bit axes inside a mask word are done in one kernel
  uint32_t pass_axis[16], n_axes = 0;
  for (uint32_t q = 0; q < g.ndim; q++) {
    const uint32_t a = c.merge_order[q];
    if (a != a0 && g.ext[a] > 1) pass_axis[n_axes++] = a;
  }
  uint32_t n_generic = n_axes;
  // (a power-of-two stride: the coordinate on the axis is then one bit of the cell index, which
  // the kernel relies on; behind an axis of another extent, e.g. a memory bound, it is not.  Not a
  // size axis: along those the cost list compares costs per volume, which that kernel does not)
  auto tail_axis = [&](uint32_t a) { return a >= 4 && g.ext[a] == 2 && g.stride[a] <= 32 && (g.stride[a] & (g.stride[a] - 1)) == 0; };
  while (n_generic > 0 && n_axes - n_generic < 6 && tail_axis(pass_axis[n_generic - 1])) n_generic--;
  TailAxes tail;
  tail.n = n_axes - n_generic;
  for (uint32_t k = 0; k < tail.n; k++) { tail.axis[k] = pass_axis[n_generic + k]; tail.stride[k] = g.stride[pass_axis[n_generic + k]]; }

  auto one_pass = [&](int which) {
    ListWork& W = LW[which];
    const uint32_t a = pass_axis[W.q_next++];
    launch_axis_pass(g, a, ++W.stamp, which == 1, W.n, W.old_alive, W.remap, W.bcell, W.blen, W.alive, W.next,
                     W.block_linked, maskL[which], prefL[which], tab->d_cost, tab->d_arg, axis_sizes(a), stL[which]);
  };
  // first part: the boxes of pass 0 and the first generic pass, then (large lists) the compaction;
  // the count of live boxes is fetched while the other list's first part runs
  bool compacted[2] = {false, false};
  for (int which = 1; which >= 0; which--) {
    ListWork& W = LW[which];
    const uint64_t nb = nbL[which];
    char* w = which == 0 ? work_lo : work_lo + wbL[0];
    W.bcell = (uint32_t*)w; w += align_up(nb * 4);
    W.blen = w; w += align_up(nb * 16);
    W.alive = (uint8_t*)w; w += align_up(nb);
    W.next = (uint32_t*)w; w += align_up(nb * 4);
    W.pos = (uint32_t*)w; w += align_up(nb * 4);
    W.cell2 = (uint32_t*)w; w += align_up(nb * 4);
    W.pos2 = (uint32_t*)w; w += align_up(nb * 4);
    W.len2 = w; w += align_up(nb * 16);
    W.alive2 = (uint8_t*)w; w += align_up(nb);
    W.block_linked = (uint32_t*)w;
    W.d_cnt = d_tot + 4 + which * 4;       // [0]: live boxes at the compaction; [2]: the final count
    W.n = (uint32_t)nb;
    launch_make_boxes(g, a0, maskL[which], prefL[which], lineL[which], colL[which], a1, W.bcell, W.blen, W.alive, stL[which]);
    if (on_cells) W.q_next = 1;               // pass_axis[0] = a1 is done
    if (W.q_next < n_generic) {
      one_pass(which);
      // (not after the pass on the cells: it leaves no dead boxes, and a compaction after the next pass costs more than it saves)
      if (!on_cells && W.n > (1u << 20) && (W.q_next < n_generic || tail.n)) {
        scan_flags(W.alive, W.n, tileL[which], W.pos, W.d_cnt, stL[which]);
        launch_compact_boxes(W.n, W.alive, W.pos, W.bcell, W.blen, W.cell2, W.len2, W.alive2, stL[which]);
        HIP_TRY(hipMemcpyAsync(aux->h_counts + 2 + which, W.d_cnt, 4, hipMemcpyDeviceToHost, stL[which]));
        compacted[which] = true;
      }
    }
  }
  // second part: the other passes on the dense arrays, the final count
  for (int which = 1; which >= 0; which--) {
    ListWork& W = LW[which];
    if (compacted[which]) {
      HIP_TRY(hipStreamSynchronize(stL[which]));
      W.n = aux->h_counts[2 + which];
      W.old_alive = W.alive; W.remap = W.pos;
      W.bcell = W.cell2; W.blen = W.len2; W.alive = W.alive2; W.pos = W.pos2;
    }
    while (W.q_next < n_generic) one_pass(which);
    if (tail.n)
      launch_tail_pairs(tail, which == 1, f.n_words, maskL[which], prefL[which], W.old_alive, W.remap, W.blen, W.alive,
                        tab->d_cost, tab->d_arg, stL[which]);
    scan_flags(W.alive, W.n, tileL[which], W.pos, W.d_cnt + 2, stL[which]);
    HIP_TRY(hipMemcpyAsync(aux->h_counts + which, W.d_cnt + 2, 4, hipMemcpyDeviceToHost, stL[which]));
    HIP_TRY(hipEventRecord(aux->events[ev_used + which], stL[which]));
  }
  // the final lists: the decisions' first (the shorter list, as a rule through first); the host
  // sleeps until a list's count has arrived
  const hipEvent_t counted[2] = {aux->events[ev_used], aux->events[ev_used + 1]};
  ev_used += 2;
  for (int which = 0; which < 2; which++) {
    const int left = 1 - which;
    HIP_TRY(hipEventSynchronize(counted[which]));
    const uint64_t nf = aux->h_counts[which];
    const size_t fb = final_bytes(nf);
    if (front + fb > (size_t)(work_lo - base)) {
      return fail(MRL_E_NOMEM, "scratch buffer too small: %zu bytes given, %zu needed", scratch_bytes,
                  front + fb + (left ? final_bytes(nbL[1 - which]) : 0) + wbL[0] + wbL[1]);
    }
    char* r = base + front;
    uint32_t* fcell = (uint32_t*)r; r += align_up(nf * 4);
    char* flen = r; r += align_up(nf * 16);
    uint64_t* fv0 = (uint64_t*)r; r += align_up(nf * 8);
    uint64_t* fv1 = (uint64_t*)r;
    const ListWork& W = LW[which];
    launch_emit(g, d_P, which == 1, W.n, W.bcell, W.blen, W.alive, W.pos, tab->d_cost, tab->d_arg, fcell, flen, fv0, fv1,
                stL[which]);
    tab->list_off[which] = front;
    tab->list_n[which] = nf;
    front += fb;
  }
  needed = front + wbL[0] + wbL[1];
  HIP_TRY(hipEventRecord(aux->events[ev_used], s2));
  HIP_TRY(hipStreamWaitEvent(st, aux->events[ev_used++], 0));
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipEventRecord(ev[2], st));
  Counters h_ctr;
  HIP_TRY(hipMemcpyAsync(&h_ctr, d_ctr, sizeof h_ctr, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (h_ctr.overflow & 2u) return fail(MRL_E_HIP, "internal error: a work item exceeded its LDS slice");
  if (h_ctr.overflow) return fail(MRL_E_OVERFLOW, "a finite cost reached 2^62");
  if (stats) {
    memset(stats, 0, sizeof *stats);
    stats->n_specs = c.n_specs;
    stats->n_admissible = stats->n_rewrites = 0;
    for (uint32_t i = 0; i < kCtrSlots; i++) { stats->n_admissible += h_ctr.n_admissible[i]; stats->n_rewrites += h_ctr.n_rewrites[i]; }
    if (P.bounded) stats->n_admissible = c.n_specs;      // no admissibility test: every Spec is evaluated
    stats->n_levels_run = n_lev;
    HIP_TRY(hipEventElapsedTime(&stats->fill_ms, ev[0], ev[1]));
    if (prefill_timed && levels_timed && deps_late) {
      // without the time the levels waited for the tables they read: work lists and pre-fill, then the levels
      float a = 0, b = 0;
      HIP_TRY(hipEventElapsedTime(&a, ev[0], ev[4]));
      HIP_TRY(hipEventElapsedTime(&b, ev[5], ev[1]));
      stats->fill_ms = a + b;
    }
    HIP_TRY(hipEventElapsedTime(&stats->compress_ms, ev[3], ev[2]));
    if (prefill_timed) HIP_TRY(hipEventElapsedTime(&stats->prefill_ms, ev[0], ev[4]));
    stats->n_decision_boxes = tab->list_n[0];
    stats->n_cost_boxes = tab->list_n[1];
    stats->scratch_used = needed;
  }
  guard.p = nullptr;
  *out = tab;
  return MRL_OK;
  });
}

}  // namespace

extern "C" {

int32_t mrl_solve(const mrl_target* t, const mrl_lattice_desc* lat, const mrl_table* const* deps, uint32_t n_deps,
                  void* d_cost, void* d_argmin, void* d_scratch, size_t scratch_bytes, void* hip_stream,
                  mrl_table** out, mrl_stats* stats) {
  return solve_impl(t, lat, deps, n_deps, d_cost, d_argmin, d_scratch, scratch_bytes, hip_stream, out, stats, FilledFn());
}

int32_t mrl_solve_graph(const mrl_target* t, const mrl_job* jobs, uint32_t n_jobs, mrl_table** out, mrl_stats* stats) {
  return guarded([&]() -> int32_t {
  if (!out) return fail(MRL_E_INVAL, "out is NULL");
  for (uint32_t j = 0; j < n_jobs && j < MRL_MAX_JOBS; j++) out[j] = nullptr;
  if (!t || !jobs) return fail(MRL_E_INVAL, "NULL argument");
  if (n_jobs < 1 || n_jobs > MRL_MAX_JOBS) return fail(MRL_E_INVAL, "n_jobs must be 1..%d", MRL_MAX_JOBS);
  for (uint32_t j = 0; j < n_jobs; j++) {
    if (!jobs[j].lattice) return fail(MRL_E_INVAL, "job %u: lattice descriptor is NULL", j);
    if (jobs[j].n_deps > 2) return fail(MRL_E_INVAL, "job %u: at most two deps", j);
    for (uint32_t i = 0; i < jobs[j].n_deps; i++)
      if (jobs[j].deps[i] >= j) return fail(MRL_E_INVAL, "job %u: a dep must be an earlier job", j);
    for (uint32_t k = 0; k < j; k++)
      if (jobs[k].hip_stream == jobs[j].hip_stream) return fail(MRL_E_INVAL, "jobs %u and %u share a stream", k, j);
  }
  // No lattice twice (solves of one (target, lattice) take turns for its upload image: such jobs
  // would not overlap, and nothing reads two tables of one lattice).
  CompiledPtr compiled[MRL_MAX_JOBS];
  for (uint32_t j = 0; j < n_jobs; j++) {
    const int32_t rc = get_compiled(t->d, jobs[j].lattice, compiled[j]);
    if (rc) { char msg[sizeof g_err]; snprintf(msg, sizeof msg, "%s", g_err); return fail(rc, "job %u: %s", j, msg); }
    for (uint32_t k = 0; k < j; k++)
      if (compiled[k] == compiled[j]) return fail(MRL_E_INVAL, "jobs %u and %u are the same lattice", k, j);
  }
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));

  enum { kWaiting = 0, kFilled = 1, kFailed = 2 };
  struct Shared {
    std::mutex mu;
    std::condition_variable cv;
    int state[MRL_MAX_JOBS] = {};
    mrl_table* table[MRL_MAX_JOBS] = {};      // from the moment a job's fill is queued
    hipEvent_t filled[MRL_MAX_JOBS] = {};     // recorded on the job's stream at that moment
    int32_t rc[MRL_MAX_JOBS] = {};
    bool skipped[MRL_MAX_JOBS] = {};          // not run: a dep failed
    std::string err[MRL_MAX_JOBS];
  } S;
  struct Events {
    Shared& s; uint32_t n = 0;
    ~Events() { for (uint32_t j = 0; j < n; j++) (void)hipEventDestroy(s.filled[j]); }
  } events{S};
  for (uint32_t j = 0; j < n_jobs; j++) {
    HIP_TRY(hipEventCreateWithFlags(&S.filled[j], hipEventDisableTiming));
    events.n = j + 1;
  }

  auto run_job = [&](uint32_t j) {
    const mrl_job& job = jobs[j];
    int32_t rc = MRL_OK;
    bool published = false;
    auto finish = [&](int32_t code) {
      if (code) S.err[j] = g_err;
      std::lock_guard<std::mutex> lk(S.mu);
      S.rc[j] = code;
      if (!published) { S.table[j] = out[j]; S.state[j] = code ? kFailed : kFilled; }
      S.cv.notify_all();
    };
    if (hipSetDevice(dev) != hipSuccess) { finish(fail(MRL_E_HIP, "hipSetDevice failed")); return; }
    // The tables the job reads, handed over when its fill needs them (its work lists and pre-fill
    // are queued by then): wait until their fills are queued; a dep's dense table is complete once
    // its stream has passed the recorded point.
    const LateDepsFn late_deps = [&](const mrl_table* tables[2], hipEvent_t ready[2]) -> int32_t {
      std::unique_lock<std::mutex> lk(S.mu);
      for (uint32_t i = 0; i < job.n_deps; i++) {
        const uint32_t d = job.deps[i];
        S.cv.wait(lk, [&] { return S.state[d] != kWaiting; });
        if (S.state[d] == kFailed) { S.skipped[j] = true; return fail(MRL_E_INVAL, "a dep of the job failed"); }
        tables[i] = S.table[d];
        ready[i] = S.filled[d];
      }
      return MRL_OK;
    };
    // (the job's own first kernels go to the GPU only once the fills it will read are queued: a
    // pre-fill that arrives before them fills every compute unit and holds them up)
    {
      std::unique_lock<std::mutex> lk(S.mu);
      for (uint32_t i = 0; i < job.n_deps; i++) S.cv.wait(lk, [&] { return S.state[job.deps[i]] != kWaiting; });
    }
    rc = solve_impl(t, job.lattice, nullptr, job.n_deps, job.d_cost, job.d_argmin, job.d_scratch,
                    job.scratch_bytes, job.hip_stream, &out[j], stats ? &stats[j] : nullptr,
                    [&](mrl_table* tab) {
                      if (hipEventRecord(S.filled[j], tab->stream) != hipSuccess) return false;   // published at the end instead
                      std::unique_lock<std::mutex> lk(S.mu);
                      S.table[j] = tab;
                      S.state[j] = kFilled;
                      published = true;
                      S.cv.notify_all();
                      // the compression waits until the jobs that read this table have queued their
                      // fill (or failed): its many small launches would otherwise hold up theirs
                      for (uint32_t k = j + 1; k < n_jobs; k++)
                        for (uint32_t i = 0; i < jobs[k].n_deps; i++)
                          if (jobs[k].deps[i] == j) S.cv.wait(lk, [&] { return S.state[k] != kWaiting; });
                      return true;
                    }, late_deps);
    finish(rc);
  };
  // a job always reports: its dependents wait for it
  auto run = [&](uint32_t j) {
    try { run_job(j); }
    catch (...) {
      std::lock_guard<std::mutex> lk(S.mu);
      S.rc[j] = MRL_E_NOMEM;
      if (S.state[j] == kWaiting) S.state[j] = kFailed;
      S.cv.notify_all();
    }
  };
  {
    // the last job runs on the calling thread, the others on the library's worker threads
    uint32_t pending = 0;                     // under S.mu: submitted jobs that have not ended
    bool submit_failed = false;
    for (uint32_t j = 0; j + 1 < n_jobs; j++) {
      { std::lock_guard<std::mutex> lk(S.mu); pending++; }
      try {
        workers().submit([&, j] {
          run(j);
          std::lock_guard<std::mutex> lk(S.mu);
          pending--;
          S.cv.notify_all();
        });
      } catch (...) {
        // no thread for this job: it and the jobs after it fail (those that wait for them wake up)
        std::lock_guard<std::mutex> lk(S.mu);
        pending--;
        for (uint32_t k = j; k < n_jobs; k++) { S.rc[k] = MRL_E_NOMEM; S.state[k] = kFailed; }
        S.cv.notify_all();
        submit_failed = true;
        break;
      }
    }
    if (!submit_failed) run(n_jobs - 1);
    std::unique_lock<std::mutex> lk(S.mu);
    S.cv.wait(lk, [&] { return pending == 0; });
  }
  uint32_t bad = n_jobs;
  for (uint32_t j = 0; j < n_jobs && bad == n_jobs; j++) if (S.rc[j] && !S.skipped[j]) bad = j;
  if (bad == n_jobs) return MRL_OK;
  // every table goes, also one that was shared before its own solve failed
  for (uint32_t j = 0; j < n_jobs; j++) {
    delete (S.table[j] ? S.table[j] : out[j]);
    out[j] = nullptr;
  }
  return fail(S.rc[bad], "job %u: %s", bad, S.err[bad].empty() ? "host allocation failed" : S.err[bad].c_str());
  });
}

void mrl_table_destroy(mrl_table* tab) { delete tab; }

int32_t mrl_query(const mrl_table* tab, const mrl_coord* specs, size_t n, uint64_t* cost_out, uint16_t* rewrite_out) {
  return guarded([&]() -> int32_t {
  if (!tab || (n && (!specs || !cost_out || !rewrite_out))) return fail(MRL_E_INVAL, "NULL argument");
  const Geo& g = tab->cp->geo;
  std::vector<uint64_t> idx(std::min<size_t>(n, kQueryChunk));
  char* base = tab->scratch;
  std::lock_guard<std::mutex> lock(tab->query_mu);
  for (size_t done = 0; done < n; done += kQueryChunk) {
    const uint32_t m = (uint32_t)std::min<size_t>(kQueryChunk, n - done);
    for (uint32_t i = 0; i < m; i++) {
      uint64_t x = 0;
      for (uint32_t a = 0; a < g.ndim; a++) {
        const uint32_t v = specs[done + i].x[a];
        if (v >= g.ext[a]) return fail(MRL_E_RANGE, "spec %zu: coordinate %u = %u outside [0, %u)", done + i, a, v, g.ext[a]);
        x += (uint64_t)v * g.stride[a];
      }
      idx[i] = x;
    }
    uint64_t* d_idx = (uint64_t*)(base + tab->f.q_idx);
    uint64_t* d_c = (uint64_t*)(base + tab->f.q_cost);
    uint16_t* d_a = (uint16_t*)(base + tab->f.q_arg);
    HIP_TRY(hipMemcpyAsync(d_idx, idx.data(), (size_t)m * 8, hipMemcpyHostToDevice, tab->stream));
    launch_gather(d_idx, m, tab->d_cost, tab->d_arg, d_c, d_a, tab->stream);
    HIP_TRY(hipMemcpyAsync(cost_out + done, d_c, (size_t)m * 8, hipMemcpyDeviceToHost, tab->stream));
    HIP_TRY(hipMemcpyAsync(rewrite_out + done, d_a, (size_t)m * 2, hipMemcpyDeviceToHost, tab->stream));
    HIP_TRY(hipStreamSynchronize(tab->stream));
  }
  return MRL_OK;
  });
}

// Staging of mrl_query_noalloc: linear indices in, costs and rewrite ids out.  One copy per GPU,
// held until the process ends; `scratch` itself is only a host-side name for it (not a device
// address): its address on the current device comes from hipGetSymbolAddress, once per device.
namespace {
struct NoAllocStaging {
  uint64_t idx[MRL_NOALLOC_MAX_QUERIES];
  uint64_t cost[MRL_NOALLOC_MAX_QUERIES];
  uint16_t arg[MRL_NOALLOC_MAX_QUERIES];
};
constexpr int kMaxDevices = 64;
std::mutex g_noalloc_mu;                       // calls that use the array take turns
void* g_noalloc_ptr[kMaxDevices] = {};         // the array's address per device, under g_noalloc_mu
}  // namespace
static __device__ __align__(256) unsigned char scratch[sizeof(NoAllocStaging)];

int32_t mrl_query_noalloc(const mrl_table* tab, const mrl_coord* specs, size_t n, uint64_t* cost_out, uint16_t* rewrite_out) {
  return guarded([&]() -> int32_t {
  if (!tab || (n && (!specs || !cost_out || !rewrite_out))) return fail(MRL_E_INVAL, "NULL argument");
  if (n > MRL_NOALLOC_MAX_QUERIES)
    return fail(MRL_E_INVAL, "mrl_query_noalloc takes at most %d Specs per call, %zu given", (int)MRL_NOALLOC_MAX_QUERIES, n);
  if (n == 0) return MRL_OK;
  const Geo& g = tab->cp->geo;
  uint64_t idx[MRL_NOALLOC_MAX_QUERIES];       // on the stack: nothing is allocated, on the host either
  for (size_t i = 0; i < n; i++) {
    uint64_t x = 0;
    for (uint32_t a = 0; a < g.ndim; a++) {
      const uint32_t v = specs[i].x[a];
      if (v >= g.ext[a]) return fail(MRL_E_RANGE, "spec %zu: coordinate %u = %u outside [0, %u)", i, a, v, g.ext[a]);
      x += (uint64_t)v * g.stride[a];
    }
    idx[i] = x;
  }
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(MRL_E_INVAL, "device %d: at most %d devices", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_noalloc_mu);
  if (!g_noalloc_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(MRL_E_HIP, "hipGetSymbolAddress gave no address");
    g_noalloc_ptr[dev] = p;
  }
  NoAllocStaging* d = (NoAllocStaging*)g_noalloc_ptr[dev];
  // the previous call's contents are simply overwritten: the kernel reads idx[0, n) and writes
  // cost[0, n), arg[0, n), and only those come back
  const uint32_t m = (uint32_t)n;
  HIP_TRY(hipMemcpyAsync(d->idx, idx, n * 8, hipMemcpyHostToDevice, tab->stream));
  launch_gather(d->idx, m, tab->d_cost, tab->d_arg, d->cost, d->arg, tab->stream);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(cost_out, d->cost, n * 8, hipMemcpyDeviceToHost, tab->stream));
  HIP_TRY(hipMemcpyAsync(rewrite_out, d->arg, n * 2, hipMemcpyDeviceToHost, tab->stream));
  HIP_TRY(hipStreamSynchronize(tab->stream));
  return MRL_OK;
  });
}

int32_t mrl_rewrite_decode(const mrl_table* tab, uint16_t id, mrl_rewrite* out) {
  return guarded([&]() -> int32_t {
  if (!tab || !out) return fail(MRL_E_INVAL, "NULL argument");
  const DevParams& P = tab->P;
  memset(out, 0, sizeof *out);
  if (id < P.move_base) { out->cls = 0; out->mk_index = id; return MRL_OK; }
  if (id < P.tile_base) {
    uint32_t r = id - P.move_base;
    out->cls = 1; out->convert = r & 1; r >>= 1;
    out->transposed = (uint8_t)(r % P.xw); r /= P.xw;
    out->dst_level = (uint8_t)(r % (P.NL - 1)); out->operand_or_dim = (uint8_t)(r / (P.NL - 1));
    return MRL_OK;
  }
  if (id < P.buf_id) {
    const uint32_t r = id - P.tile_base, d = r / P.maxs, j = r % P.maxs;
    if (j >= P.nsz[d]) return fail(MRL_E_RANGE, "rewrite id %u names no tile size", id);
    out->cls = 2; out->operand_or_dim = (uint8_t)d; out->tile_size = tab->cp->sizes[d][j];
    return MRL_OK;
  }
  if (id == P.buf_id && P.kind == kKindF) { out->cls = 3; return MRL_OK; }
  if (P.split && id >= P.buf_id && id < P.buf_id + P.NL) { out->cls = 3; out->dst_level = (uint8_t)(id - P.buf_id); return MRL_OK; }
  if (P.par && id >= P.par_base && id < P.par_base + 4 * P.maxs) {
    const uint32_t r = id - P.par_base, d = r / P.maxs, j = r % P.maxs;
    if (d != 2 && j < P.nsz[d]) { out->cls = 4; out->operand_or_dim = (uint8_t)d; out->tile_size = P.sizes[d][j]; return MRL_OK; }
  }
  return fail(MRL_E_RANGE, "rewrite id %u is not used by this table", id);
  });
}

int32_t mrl_coord_of_spec(const mrl_table* tab, const uint32_t shape[4], const uint8_t* levels, const uint8_t* layouts,
                          const uint8_t* dtypes, mrl_coord* out) {
  return guarded([&]() -> int32_t {
  if (!tab || !shape || !levels || !out) return fail(MRL_E_INVAL, "NULL argument");
  const Compiled& c = *tab->cp;
  memset(out, 0, sizeof *out);
  for (int d = 0; d < 4; d++) {
    auto it = std::lower_bound(c.sizes[d].begin(), c.sizes[d].end(), shape[d]);
    if (it == c.sizes[d].end() || *it != shape[d]) return fail(MRL_E_RANGE, "size %u is not allowed on dimension %d", shape[d], d);
    out->x[d] = (uint32_t)(it - c.sizes[d].begin());
  }
  for (uint32_t i = 0; i < c.P.nlv; i++) {
    if (levels[i] >= c.P.NL) return fail(MRL_E_RANGE, "level %u of operand %u outside the target", levels[i], i);
    out->x[4 + i] = levels[i];
  }
  for (uint32_t a = 0; a < c.P.nlim; a++) out->x[4 + c.P.nlv + a] = c.P.lim_nq[a] - 1;   // the whole capacity
  for (uint32_t i = 0; i < c.P.nops; i++) {
    if (c.lay_axis[i] >= 0) { if (!layouts || layouts[i] >= (1u << c.P.lay_w[i])) return fail(MRL_E_RANGE, "layout of operand %u", i); out->x[c.lay_axis[i]] = layouts[i]; }
    if (c.dt_axis[i] >= 0) { if (!dtypes || dtypes[i] > 1) return fail(MRL_E_RANGE, "dtype of operand %u", i); out->x[c.dt_axis[i]] = dtypes[i]; }
  }
  return MRL_OK;
  });
}

int32_t mrl_schedule(const mrl_table* tab, const mrl_coord* goal, mrl_schedule_node* out, size_t cap, size_t* n_out) {
  return guarded([&]() -> int32_t {
  if (!tab || !goal) return fail(MRL_E_INVAL, "NULL argument");
  struct Item { const mrl_table* t; uint32_t which; mrl_coord x; };
  std::vector<Item> stack;
  stack.push_back({tab, 0u, *goal});
  size_t n = 0;
  while (!stack.empty()) {
    const Item it = stack.back();
    stack.pop_back();
    const Compiled& c = *it.t->cp;
    const DevParams& P = it.t->P;
    uint64_t cost;
    uint16_t rw;
    int32_t rc = mrl_query(it.t, &it.x, 1, &cost, &rw);
    if (rc) return rc;
    if (cost == kInf) {
      if (n == 0) return fail(MRL_E_INVAL, "the goal Spec has no implementation");
      return fail(MRL_E_HIP, "internal error: a rewrite of a finite Spec leads to a Spec without implementation");
    }
    mrl_rewrite r;
    rc = mrl_rewrite_decode(it.t, rw, &r);
    if (rc) return rc;
    mrl_schedule_node node;
    memset(&node, 0, sizeof node);
    node.table = it.which; node.rewrite = rw; node.cost = cost; node.spec = it.x;
    if (r.cls == 1) {                       // Move: the operand one or more levels down, perhaps in another layout / converted
      const uint32_t op = r.operand_or_dim;
      Item ch = it;
      ch.x.x[4 + op] = r.dst_level;
      if (r.transposed) { if (c.lay_axis[op] < 0) return fail(MRL_E_HIP, "internal error: transposing Move without a layout coordinate"); ch.x.x[c.lay_axis[op]] ^= r.transposed; }
      if (r.convert) { if (c.dt_axis[op] < 0) return fail(MRL_E_HIP, "internal error: converting Move without a dtype coordinate"); ch.x.x[c.dt_axis[op]] = 0; }
      if (P.bounded && P.lim_of_level[r.dst_level] != kNoBit) {
        // the Move's buffer comes out of the destination's bound; the rest snaps down to a power of two
        const uint32_t ax = 4 + P.nlv + P.lim_of_level[r.dst_level];
        const uint64_t b = c.sizes[0][it.x.x[0]], m = c.sizes[1][it.x.x[1]], k = c.sizes[2][it.x.x[2]], nn = c.sizes[3][it.x.x[3]];
        const uint64_t numel = P.kind == kKindM ? (op == 0 ? b * m * k : op == 1 ? b * k * nn : b * m * nn)
                             : P.kind == kKindE ? (op == 1 ? nn : m * nn)
                                                : (op == 0 ? m * k : op == 1 ? k * nn : op == 2 ? nn : m * nn);
        const bool bf = c.dt_axis[op] >= 0 ? ch.x.x[c.dt_axis[op]] != 0 : c.lat.base_dtype_bytes[op] == 2;
        const uint64_t bytes = numel * (bf ? 2 : 4), have = it.x.x[ax] ? 1ull << (it.x.x[ax] - 1) : 0;
        if (bytes > have) return fail(MRL_E_HIP, "internal error: a memoized Move exceeds its memory bound");
        uint64_t left = have - bytes;
        uint32_t q = 0;
        while (left) { q++; left >>= 1; }
        ch.x.x[ax] = q;
      }
      node.n_children = 1;
      if (P.moves) {
        // Section 2, Memory Movement: the alloc-binding holds a load Move Spec (operands that are read),
        // the body, and a store Move Spec (operands that are written), both of fresh tensors
        if (it.which != 0 || !it.t->deps[0]) return fail(MRL_E_HIP, "internal error: a Move Spec outside a MATMUL_MOVES table");
        const mrl_table* vt = it.t->deps[0];
        const Compiled& vc = *vt->cp;
        const uint32_t y0 = c.lay_axis[op] >= 0 ? it.x.x[c.lay_axis[op]] : 0u, y1 = c.lay_axis[op] >= 0 ? ch.x.x[c.lay_axis[op]] : 0u;
        const uint32_t f0 = c.dt_axis[op] >= 0 ? it.x.x[c.dt_axis[op]] : (uint32_t)(c.lat.base_dtype_bytes[op] == 2);
        const uint32_t f1 = c.dt_axis[op] >= 0 ? ch.x.x[c.dt_axis[op]] : f0;
        auto move_spec = [&](uint32_t ls, uint32_t ld, uint32_t ys, uint32_t yd, uint32_t fs, uint32_t fd, Item& out_item) -> int32_t {
          out_item = Item{vt, 1u, {}};
          mrl_coord& x = out_item.x;
          memset(&x, 0, sizeof x);
          x.x[1] = op == 1 ? it.x.x[2] : it.x.x[1];      // rows: m (lhs, out) or k (rhs); the size lists are the same
          x.x[3] = op == 0 ? it.x.x[2] : it.x.x[3];      // columns: k (lhs) or n
          x.x[4] = ls; x.x[5] = ld;
          x.x[6] = ys >= 2 ? 3 : 2; x.x[7] = 1; x.x[8] = yd >= 2 ? 3 : 2; x.x[9] = 1;
          if (vc.lay_axis[0] >= 0) x.x[vc.lay_axis[0]] = ys; else if (ys) return fail(MRL_E_HIP, "internal error: the MOVE table lacks a layout coordinate");
          if (vc.lay_axis[1] >= 0) x.x[vc.lay_axis[1]] = yd; else if (yd) return fail(MRL_E_HIP, "internal error: the MOVE table lacks a layout coordinate");
          if (vc.dt_axis[0] >= 0) x.x[vc.dt_axis[0]] = fs;
          if (vc.dt_axis[1] >= 0) x.x[vc.dt_axis[1]] = fd;
          return MRL_OK;
        };
        Item load, store;
        const bool has_load = P.access[op] != kWrite, has_store = P.access[op] != kRead;
        if (has_store) { rc = move_spec(r.dst_level, it.x.x[4 + op], y1, y0, f1, f0, store); if (rc) return rc; stack.push_back(store); }
        stack.push_back(ch);                // popped after the load's whole subtree, before the store's
        if (has_load) { rc = move_spec(it.x.x[4 + op], r.dst_level, y0, y1, f0, f1, load); if (rc) return rc; stack.push_back(load); }
        node.n_children = (uint16_t)(1 + (has_load ? 1 : 0) + (has_store ? 1 : 0));
      } else {
        stack.push_back(ch);
      }
    } else if (r.cls == 2) {                // tile: the loop body is the Spec with the smaller size
      const uint32_t d = r.operand_or_dim, j = (rw - P.tile_base) % P.maxs;
      Item ch = it;
      ch.x.x[d] = j;
      if (P.kind == kKindV) {
        // Section 2.4.3: what is known of the tile of either tensor
        const uint32_t rows = c.sizes[1][it.x.x[1]], cols = c.sizes[3][it.x.x[3]];
        const uint32_t r2 = c.sizes[1][ch.x.x[1]], c2 = c.sizes[3][ch.x.x[3]];
        for (int ts = 0; ts < 2; ts++) {
          const uint32_t y = c.lay_axis[ts] >= 0 ? it.x.x[c.lay_axis[ts]] : 0u;
          const bool bf = c.dt_axis[ts] >= 0 ? it.x.x[c.dt_axis[ts]] != 0 : c.lat.base_dtype_bytes[ts] == 2;
          uint32_t contig2, aligned2;
          tile_abstract(y, rows, cols, r2, c2, bf ? 2 : 4, P.strip ? P.strip : 1, P.line_bytes, P.line_mask, it.x.x[6 + 2 * ts], it.x.x[7 + 2 * ts],
                        contig2, aligned2);
          ch.x.x[6 + 2 * ts] = contig2; ch.x.x[7 + 2 * ts] = aligned2;
        }
      }
      stack.push_back(ch);
      node.n_children = 1;
    } else if (r.cls == 4) {                // parallel loop: the body is the serial-only Spec of the smaller size
      if (it.which != 0 || !it.t->deps[0]) return fail(MRL_E_HIP, "internal error: parallel loop outside a MATMUL_PARALLEL table");
      const uint32_t d = r.operand_or_dim, j = (rw - P.par_base) % P.maxs;
      Item ch{it.t->deps[0], 1u, it.x};
      ch.x.x[d] = j;
      stack.push_back(ch);
      node.n_children = 1;
    } else if (r.cls == 3 && P.split) {     // bufferize between the bias add and the ReLU, the intermediate in level r.dst_level
      if ((it.which != 0 && it.which != 2) || !it.t->deps[0] || !it.t->deps[1]) return fail(MRL_E_HIP, "internal error: bufferize outside a BIAS_ADD_RELU_SPLIT table");
      const uint32_t m = c.sizes[1][it.x.x[1]], nn = c.sizes[3][it.x.x[3]];
      const uint8_t l_mid = r.dst_level;
      const uint8_t y_in = c.lay_axis[0] >= 0 ? (uint8_t)it.x.x[c.lay_axis[0]] : 0, y_out = c.lay_axis[2] >= 0 ? (uint8_t)it.x.x[c.lay_axis[2]] : 0;
      const uint32_t shape_e[4] = {1, m, 1, nn};
      const uint8_t lv_a[5] = {(uint8_t)it.x.x[4], (uint8_t)it.x.x[5], l_mid, 0, 0}, ly_a[5] = {y_in, 0, 0, 0, 0};
      const uint8_t lv_r[5] = {l_mid, (uint8_t)it.x.x[6], 0, 0, 0}, ly_r[5] = {0, y_out, 0, 0, 0};
      const uint8_t zeros[5] = {0, 0, 0, 0, 0};
      // (tables 3 and 4 when this table is itself dep 1 of the table the walk started in)
      Item ca{it.t->deps[0], it.which + 1u, {}}, cr{it.t->deps[1], it.which + 2u, {}};
      rc = mrl_coord_of_spec(ca.t, shape_e, lv_a, ly_a, zeros, &ca.x);
      if (rc) return rc;
      rc = mrl_coord_of_spec(cr.t, shape_e, lv_r, ly_r, zeros, &cr.x);
      if (rc) return rc;
      stack.push_back(cr);                  // popped after the bias add's whole subtree
      stack.push_back(ca);
      node.n_children = 2;
    } else if (r.cls == 3 && P.chain) {     // bufferize of a composition: the Matmul (m, k, p) into the intermediate, then (m, p, n) out of it
      if (it.which != 0 || !it.t->deps[0]) return fail(MRL_E_HIP, "internal error: bufferize outside a MATMUL_CHAIN table");
      const uint32_t p = c.sizes[0][it.x.x[0]], m = c.sizes[1][it.x.x[1]], k = c.sizes[2][it.x.x[2]], nn = c.sizes[3][it.x.x[3]];
      const uint8_t l_mid = (uint8_t)it.x.x[8];
      uint8_t y[4];
      for (int i = 0; i < 4; i++) y[i] = c.lay_axis[i] >= 0 ? (uint8_t)it.x.x[c.lay_axis[i]] : 0;
      const uint32_t shape_1[4] = {1, m, k, p}, shape_2[4] = {1, m, p, nn};
      const uint8_t lv_1[5] = {(uint8_t)it.x.x[4], (uint8_t)it.x.x[5], l_mid, 0, 0}, ly_1[5] = {y[0], y[1], 0, 0, 0};
      const uint8_t lv_2[5] = {l_mid, (uint8_t)it.x.x[6], (uint8_t)it.x.x[7], 0, 0}, ly_2[5] = {0, y[2], y[3], 0, 0};
      const uint8_t zeros[5] = {0, 0, 0, 0, 0};
      Item c1{it.t->deps[0], 1u, {}}, c2{it.t->deps[0], 1u, {}};
      rc = mrl_coord_of_spec(c1.t, shape_1, lv_1, ly_1, zeros, &c1.x);
      if (rc) return rc;
      rc = mrl_coord_of_spec(c2.t, shape_2, lv_2, ly_2, zeros, &c2.x);
      if (rc) return rc;
      stack.push_back(c2);                  // popped after the first Matmul's whole subtree
      stack.push_back(c1);
      node.n_children = 2;
    } else if (r.cls == 3) {                // bufferize: Matmul into the intermediate, then bias-add + ReLU out of it
      if (it.which != 0 || !it.t->deps[0] || !it.t->deps[1]) return fail(MRL_E_HIP, "internal error: bufferize outside a FUSED table");
      const uint32_t m = c.sizes[1][it.x.x[1]], k = c.sizes[2][it.x.x[2]], nn = c.sizes[3][it.x.x[3]];
      const uint8_t l_lhs = (uint8_t)it.x.x[4], l_rhs = (uint8_t)it.x.x[5], l_bias = (uint8_t)it.x.x[6], l_out = (uint8_t)it.x.x[7];
      const uint8_t l_mid = (uint8_t)it.x.x[8];
      const uint8_t y_lhs = c.lay_axis[0] >= 0 ? (uint8_t)it.x.x[c.lay_axis[0]] : 0, y_rhs = c.lay_axis[1] >= 0 ? (uint8_t)it.x.x[c.lay_axis[1]] : 0;
      const uint8_t y_out = c.lay_axis[3] >= 0 ? (uint8_t)it.x.x[c.lay_axis[3]] : 0;
      const uint32_t shape_m[4] = {1, m, k, nn}, shape_e[4] = {1, m, 1, nn};
      const uint8_t lv_m[5] = {l_lhs, l_rhs, l_mid, 0, 0}, ly_m[5] = {y_lhs, y_rhs, 0, 0, 0};
      const uint8_t lv_e[5] = {l_mid, l_bias, l_out, 0, 0}, ly_e[5] = {0, 0, y_out, 0, 0};
      const uint8_t zeros[5] = {0, 0, 0, 0, 0};
      Item cm{it.t->deps[0], 1u, {}}, ce{it.t->deps[1], 2u, {}};
      rc = mrl_coord_of_spec(cm.t, shape_m, lv_m, ly_m, zeros, &cm.x);
      if (rc) return rc;
      rc = mrl_coord_of_spec(ce.t, shape_e, lv_e, ly_e, zeros, &ce.x);
      if (rc) return rc;
      if (P.bounded) {
        // both stages inherit the bounds; the intermediate's bytes come out of its level's bound
        for (uint32_t a = 0; a < P.nlim; a++) cm.x.x[4 + 3 + a] = ce.x.x[4 + 3 + a] = it.x.x[4 + P.nlv + a];
        if (P.lim_of_level[l_mid] != kNoBit) {
          const uint32_t a = P.lim_of_level[l_mid], q = it.x.x[4 + P.nlv + a];
          const uint64_t bytes = (uint64_t)m * nn * 4, have = q ? 1ull << (q - 1) : 0;
          if (bytes > have) return fail(MRL_E_HIP, "internal error: a memoized bufferize exceeds its memory bound");
          uint64_t left = have - bytes;
          uint32_t qn = 0;
          while (left) { qn++; left >>= 1; }
          cm.x.x[4 + 3 + a] = ce.x.x[4 + 3 + a] = qn;
        }
      }
      stack.push_back(ce);                  // popped after the Matmul's whole subtree
      stack.push_back(cm);
      node.n_children = 2;
    }
    if (out && n < cap) out[n] = node;
    n++;
    if (n > (1u << 20)) return fail(MRL_E_HIP, "internal error: schedule does not end");
  }
  if (n_out) *n_out = n;
  if (out && cap < n) return fail(MRL_E_BUFSZ, "schedule buffer holds %zu nodes, %zu needed", cap, n);
  return MRL_OK;
  });
}

int32_t mrl_emit_compressed(const mrl_table* tab, uint32_t which, mrl_box* out, size_t cap, size_t* n_out) {
  return guarded([&]() -> int32_t {
  if (!tab || which > 1) return fail(MRL_E_INVAL, "bad argument");
  const uint64_t n = tab->list_n[which];
  if (n_out) *n_out = n;
  if (!out) return MRL_OK;
  if (cap < n) return fail(MRL_E_BUFSZ, "box buffer holds %zu, %llu needed", cap, (unsigned long long)n);
  const Geo& g = tab->cp->geo;
  const char* r = tab->scratch + tab->list_off[which];
  std::vector<uint32_t> fcell(n);
  std::vector<uint8_t> flen(n * 16);
  std::vector<uint64_t> fv0(n), fv1(n);
  if (n) {
    HIP_TRY(hipMemcpy(fcell.data(), r, n * 4, hipMemcpyDeviceToHost)); r += align_up(n * 4);
    HIP_TRY(hipMemcpy(flen.data(), r, n * 16, hipMemcpyDeviceToHost)); r += align_up(n * 16);
    HIP_TRY(hipMemcpy(fv0.data(), r, n * 8, hipMemcpyDeviceToHost)); r += align_up(n * 8);
    HIP_TRY(hipMemcpy(fv1.data(), r, n * 8, hipMemcpyDeviceToHost));
  }
  for (uint64_t i = 0; i < n; i++) {
    mrl_box& b = out[i];
    memset(&b, 0, sizeof b);
    uint32_t x = fcell[i];
    for (uint32_t a = 0; a < g.ndim; a++) {
      const uint32_t lo = x / g.stride[a];
      x -= lo * g.stride[a];
      b.lo[a] = (uint16_t)lo;
      b.hi[a] = (uint16_t)(lo + flen[i * 16 + a] - 1);
    }
    b.v0 = fv0[i]; b.v1 = fv1[i];
  }
  return MRL_OK;
  });
}

int32_t mrl_query_compressed(const mrl_table* tab, const mrl_coord* specs, size_t n, uint64_t* cost_out,
                             uint16_t* rewrite_out) {
  return guarded([&]() -> int32_t {
  if (!tab || (n && (!specs || !cost_out || !rewrite_out))) return fail(MRL_E_INVAL, "NULL argument");
  const Compiled& c = *tab->cp;
  const Geo& g = c.geo;
  for (uint32_t a = 0; a < g.ndim; a++)
    if (g.ext[a] > 256) return fail(MRL_E_INVAL, "axis %u has %u coordinates: the box index holds one byte per axis", a, g.ext[a]);
  std::lock_guard<std::mutex> lock(tab->lookup_mu);
  const uint64_t* fv[2][2];
  const uint32_t* cells[2];
  for (uint32_t which = 0; which < 2; which++) {
    const uint64_t nb = tab->list_n[which];
    const char* r = tab->scratch + tab->list_off[which];
    const uint32_t* fcell = cells[which] = (const uint32_t*)r; r += align_up(nb * 4);
    const void* flen = r; r += align_up(nb * 16);
    fv[which][0] = (const uint64_t*)r; r += align_up(nb * 8);
    fv[which][1] = (const uint64_t*)r;
    mrl_table::BoxIndex& ix = tab->index[which];
    if (!ix.nodes) {
      ix.L = index_levels((uint32_t)nb);
      HIP_TRY(hipMalloc((void**)&ix.nodes, std::max<size_t>(ix.L.total, 1) * sizeof(BoxBounds)));
      launch_build_index(g, ix.L, fcell, flen, ix.nodes, tab->stream);
      HIP_TRY(hipGetLastError());
    }
  }
  // staging of one chunk: points, then per list v0, v1 (u64) and the box index (u32)
  const size_t o_pts = 0, o_val = o_pts + (size_t)kLookupChunk * 16, o_which = o_val + 4 * (size_t)kLookupChunk * 8,
               total = o_which + 2 * (size_t)kLookupChunk * 4;
  if (!tab->lookup_buf) HIP_TRY(hipMalloc((void**)&tab->lookup_buf, total));
  uint8_t* d_pts = (uint8_t*)(tab->lookup_buf + o_pts);
  uint64_t* d_val = (uint64_t*)(tab->lookup_buf + o_val);
  uint32_t* d_which = (uint32_t*)(tab->lookup_buf + o_which);
  std::vector<uint8_t> pts((size_t)kLookupChunk * 16);
  std::vector<uint64_t> val(4 * (size_t)kLookupChunk), vol(kLookupChunk);
  std::vector<uint32_t> hit(2 * (size_t)kLookupChunk);
  for (size_t done = 0; done < n; done += kLookupChunk) {
    const uint32_t m = (uint32_t)std::min<size_t>(kLookupChunk, n - done);
    memset(pts.data(), 0, (size_t)m * 16);
    for (uint32_t i = 0; i < m; i++) {
      for (uint32_t a = 0; a < g.ndim; a++) {
        const uint32_t v = specs[done + i].x[a];
        if (v >= g.ext[a]) return fail(MRL_E_RANGE, "spec %zu: coordinate %u = %u outside [0, %u)", done + i, a, v, g.ext[a]);
        pts[(size_t)i * 16 + a] = (uint8_t)v;
      }
      uint64_t w = 1;
      for (uint32_t d = 0; d < 4; d++) w *= c.sizes[d][specs[done + i].x[d]];
      vol[i] = w;
    }
    HIP_TRY(hipMemcpyAsync(d_pts, pts.data(), (size_t)m * 16, hipMemcpyHostToDevice, tab->stream));
    for (uint32_t which = 0; which < 2; which++)
      launch_lookup(g, tab->index[which].L, tab->index[which].nodes, cells[which], d_pts, m, fv[which][0], fv[which][1],
                    d_val + (2 * which) * (size_t)kLookupChunk, d_val + (2 * which + 1) * (size_t)kLookupChunk,
                    d_which + which * (size_t)kLookupChunk, tab->stream);
    HIP_TRY(hipGetLastError());
    for (uint32_t k = 0; k < 4; k++)
      HIP_TRY(hipMemcpyAsync(val.data() + k * (size_t)kLookupChunk, d_val + k * (size_t)kLookupChunk, (size_t)m * 8,
                             hipMemcpyDeviceToHost, tab->stream));
    for (uint32_t k = 0; k < 2; k++)
      HIP_TRY(hipMemcpyAsync(hit.data() + k * (size_t)kLookupChunk, d_which + k * (size_t)kLookupChunk, (size_t)m * 4,
                             hipMemcpyDeviceToHost, tab->stream));
    HIP_TRY(hipStreamSynchronize(tab->stream));
    for (uint32_t i = 0; i < m; i++) {
      if (hit[i] == 0xFFFFFFFFu || hit[kLookupChunk + i] == 0xFFFFFFFFu)
        return fail(MRL_E_HIP, "internal error: spec %zu lies in no box", done + i);
      rewrite_out[done + i] = (uint16_t)val[i];
      const uint64_t v0 = val[2 * (size_t)kLookupChunk + i], v1 = val[3 * (size_t)kLookupChunk + i];
      cost_out[done + i] = v1 == 0 ? kInf : (uint64_t)((unsigned __int128)v0 * vol[i] / v1);
    }
  }
  return MRL_OK;
  });
}

int32_t mrl_copy_dense(const mrl_table* tab, uint64_t* cost_host, uint16_t* argmin_host) {
  return guarded([&]() -> int32_t {
  if (!tab) return fail(MRL_E_INVAL, "table is NULL");
  if (cost_host) HIP_TRY(hipMemcpy(cost_host, tab->d_cost, tab->cp->n_specs * 8, hipMemcpyDeviceToHost));
  if (argmin_host) HIP_TRY(hipMemcpy(argmin_host, tab->d_arg, tab->cp->n_specs * 2, hipMemcpyDeviceToHost));
  return MRL_OK;
  });
}

}  // extern "C"
