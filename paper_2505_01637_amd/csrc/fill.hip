// Rewrite evaluation + argmin for one dependency level of the Spec lattice.
//
// Paper, Section 4: a Spec's entry is the lowest-cost applicable rewrite, the
// rewrite's cost being the affine function of Section 3 of its sub-Specs'
// costs.  Here the table is filled bottom-up: all shapes of one dependency
// level in one launch, every sub-Spec of another shape already final.
//
// Mapping (gfx950, wave64).  One wavefront owns one shape (b,m,k,n): all its
// level / layout / dtype entries, which is a set closed under Moves, so waves
// never wait for each other and the wave's writes are one contiguous stretch
// of the table.  Per shape:
//   1. lanes decide, per level assignment, which entries fit their levels;
//      the admissible ones are compacted, ordered by rank (sum of the operand
//      levels), into a task list in LDS (most entries do not fit);
//   2. (before the first level, once per table) the whole table is set to
//      (INF, NONE) by the plan kernel's waves (or a plain streaming kernel), so
//      this kernel writes the admissible entries only;
//   3. one lane per task evaluates the tile and bufferize rewrites, whose
//      sub-Specs belong to other shapes or tables and are final: a tile
//      sub-Spec sits at the same offset of a smaller shape's group, so
//      consecutive lanes read consecutive addresses, several loads in flight
//      per lane.  The best of them is parked in LDS;
//   4. rank by rank, one lane per task evaluates the microkernels and the
//      Moves (sub-Specs of the same shape at a lower rank: read from LDS), in
//      id order, keeping the first strict minimum (= lowest id among ties),
//      then takes the parked candidate if strictly lower (its ids are higher).
//      Results go to LDS (for later ranks) and to the table.
// Before the first level a plan kernel counts, per shape and per value of the
// passive level axis (the intermediate's level of a fused Spec: such slices are
// independent), the entries that fit, and sorts the work into three lists per
// dependency level: shapes one wave can hold whole, slices one wave can hold,
// and slices that get a whole workgroup and an LDS slice sized for the largest
// possible slice.  Shapes in which nothing fits get no work at all.  Nothing is
// reduced across lanes and no result depends on which wave handles an item:
// the table is deterministic.
#include <hip/hip_runtime.h>
#include <cstdlib>
#include "compress.h"
#include "dev_params.h"

namespace mrl {

constexpr int kBatch = 8;              // sub-Spec costs fetched together before they are compared
constexpr uint32_t kSmallCap = 512;    // entries per shape up to which a shape's whole group is one LDS slice
constexpr uint32_t kSlicedCap = 256;   // tasks per LDS slice for lattices with more entries per shape
constexpr uint32_t kWaveCap = 64;      // whole shapes of at most this many tasks count as small
constexpr uint32_t kBigBlock = 512;    // threads per item that does not fit a wave's slice
constexpr uint32_t kTileLds = 64;      // tile rewrites of the shape staged in LDS at a time
constexpr uint32_t kWideBelow = 2048;  // levels with fewer shapes than this get 256 threads per shape

struct Eval {
  uint64_t best;
  uint32_t arg;
  uint32_t n;
  uint32_t ovf;
};

// Keep the lexicographic minimum of (cost, rewrite id) among the candidates with ok set (all
// finite), so the evaluation order of the rewrites is free.  Written with selects: as branches
// the many calls cost more in exec-mask bookkeeping than the work they skip.
__device__ __forceinline__ void consider(Eval& e, uint64_t cand, uint32_t id, bool ok = true) {
  const bool better = ok & ((cand < e.best) | ((cand == e.best) & (id < e.arg)));
  e.best = better ? cand : e.best;
  e.arg = better ? id : e.arg;
}

// a * b for operands below 2^62 and 2^33; kLimit if the product reaches 2^62.
__device__ __forceinline__ uint64_t mul_or_limit(uint64_t a, uint64_t b) {
  const uint64_t lo = a * b;
  return (__umul64hi(a, b) != 0 || lo >= kLimit) ? kLimit : lo;
}

struct Shape {
  uint32_t si[4];
  uint64_t d[4];
  uint64_t numel[5];
};

__device__ __forceinline__ void load_shape(const DevParams* __restrict__ P, uint32_t shape, Shape& S) {
  uint32_t r = shape;
#pragma unroll
  for (int a = 0; a < 4; a++) {
    S.si[a] = r / P->shape_stride[a];
    r -= S.si[a] * P->shape_stride[a];
    S.d[a] = P->sizes[a][S.si[a]];
  }
  uint64_t b = S.d[0], m = S.d[1], k = S.d[2], n = S.d[3];
  if (P->kind == kKindM) { S.numel[0] = b * m * k; S.numel[1] = b * k * n; S.numel[2] = b * m * n; S.numel[3] = 0; S.numel[4] = 0; }
  else if (P->kind == kKindV) { S.numel[0] = m * n; S.numel[1] = m * n; S.numel[2] = 0; S.numel[3] = 0; S.numel[4] = 0; }
  else if (P->kind == kKindE) { S.numel[0] = m * n; S.numel[1] = n; S.numel[2] = m * n; S.numel[3] = 0; S.numel[4] = m * n; }   // [4]: the intermediate of a split
  else if (P->kind == kKindR) { S.numel[0] = m * n; S.numel[1] = m * n; S.numel[2] = 0; S.numel[3] = 0; S.numel[4] = 0; }
  else if (P->chain) { S.numel[0] = m * k; S.numel[1] = k * b; S.numel[2] = b * n; S.numel[3] = m * n; S.numel[4] = m * b; }   // b holds p
  else { S.numel[0] = m * k; S.numel[1] = k * n; S.numel[2] = n; S.numel[3] = m * n; S.numel[4] = m * n; }
}

// The uniform fields the per-task code needs, read once per unit so that they stay in scalar
// registers (a scalar load in the middle of the LDS traffic stalls on the counter they share).
struct Hot {
  uint32_t nops, NL, npass, log2V, ndt, move_base;
  uint32_t pack_shift[4], lay_bit[4], dt_bit[4], can_convert[4], lvpow[4];
  // the same per-operand fields, one byte per operand (0xFF = no bit), for lanes that pick their
  // operand by lane index: a shift instead of an indexed read (which would put the struct in scratch)
  uint32_t lay_bytes, dt_bytes, shift_bytes, cv_bits;
};

__device__ __forceinline__ Hot load_hot(const DevParams* __restrict__ P) {
  Hot H;
  H.nops = P->nops; H.NL = P->NL; H.npass = P->npass; H.log2V = P->log2V; H.ndt = P->ndt; H.move_base = P->move_base;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    H.pack_shift[i] = P->pack_shift[i]; H.lay_bit[i] = P->lay_bit[i]; H.dt_bit[i] = P->dt_bit[i];
    H.can_convert[i] = P->can_convert[i]; H.lvpow[i] = P->lvpow[i];
  }
  H.lay_bytes = H.dt_bytes = H.shift_bytes = H.cv_bits = 0;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    H.lay_bytes |= (H.lay_bit[i] == kNoBit ? 0xFFu : H.lay_bit[i] & 0xFFu) << (8 * i);
    H.dt_bytes |= (H.dt_bit[i] == kNoBit ? 0xFFu : H.dt_bit[i] & 0xFFu) << (8 * i);
    H.shift_bytes |= (H.pack_shift[i] & 0xFFu) << (8 * i);
    H.cv_bits |= (H.can_convert[i] ? 1u : 0u) << i;
  }
  return H;
}

// Table offset (inside the shape's group) of entry (pack, pass, variant).
__device__ __forceinline__ uint32_t entry_offset(const Hot& H, uint32_t xpack, uint32_t v) {
  const uint32_t pack = xpack & 0xFFu, pass = xpack >> 8;
  uint32_t combo = pack;
  if (H.NL != 4) {
    combo = 0;
#pragma unroll
    for (int i = 0; i < 4; i++) if ((uint32_t)i < H.nops) combo += ((pack >> H.pack_shift[i]) & 3u) * H.lvpow[i];
  }
  return ((combo * H.npass + pass) << H.log2V) + v;
}

// Shape part of microkernel j's predicate: number of repetitions, 0 if it fails
// (Section 2, Microkernel Selection; Figure 1 for BroadcastVecMultAdd).  The
// level/layout/dtype part is tabulated per entry (DevParams::mk_entry).
__device__ __forceinline__ uint64_t mk_shape_reps(const DevParams* __restrict__ P, const Shape& S, uint32_t j) {
  const uint64_t b = S.d[0], m = S.d[1], k = S.d[2], n = S.d[3];
  const uint32_t lanes = P->mk_lanes[j];
  switch (P->mk_kind[j]) {
    case 0: return (b == 1 && m == 1 && k == 1 && n == 1) ? 1 : 0;
    case 1: return (b == 1 && m == 1 && k == 1 && n % lanes == 0) ? n / lanes : 0;
    case 2: return (b == 1 && m == 1 && n == 1 && k % lanes == 0) ? k / lanes : 0;
    case 3: return (m == 1 && n == 1) ? 1 : 0;
    case 4: return (m == 1 && n % lanes == 0) ? n / lanes : 0;
    case 5: return (m == 1 && n == 1) ? 1 : 0;                       // Move Specs: m rows, n columns
    case 6:
    case 7: return (m == 1 && n % lanes == 0) ? n / lanes : 0;
    case 8:                                                          // bias add alone, ReLU alone: one element,
    case 10: return (m == 1 && n == 1) ? 1 : 0;
    case 9:                                                          // or one row of whole vectors
    case 11: return (m == 1 && n % lanes == 0) ? n / lanes : 0;
    default: return 0;
  }
}

// LDS of one unit (a shape, or one passive-level slice of it).  "xpack" = pass<<8 | pack.
struct UnitLds {
  uint64_t* bterm;    // [256] Move cost of this shape: [convert][operand][src][dst][transposed]; 0 = no such Move
  uint64_t* tl_base;  // [kTileLds] tile rewrites of this shape: table offset of the sub-shape's group,
  uint32_t* tl_trips; // [kTileLds]   trip count,
  uint32_t* tl_id;    // [kTileLds]   rewrite id
  uint64_t* t_cost;   // [cap] per task: best tile/bufferize candidate, then the final cost
  uint32_t* t_spec;   // [cap] xpack | variant<<10 | id<<16
  uint32_t* c_info;   // [npass*256] by xpack: admissible variants (low 16 bits) | first task << 16
  uint32_t* r_off;    // [nranks+1] first task of the rank
  uint32_t* wave_tot; // [16] scan scratch
  uint32_t* fit;      // [16] see build_fit
};

__host__ __device__ inline uint32_t unit_lds_bytes(uint32_t cap, uint32_t npass) {
  return (2048u + kTileLds * 16u + cap * 12u + npass * 1024u + (kMaxRanks + 2) * 4u + 32u * 4u + 16u + 15u) & ~15u;   // slices stay 16-byte aligned
}

__device__ __forceinline__ UnitLds carve(unsigned char* w, uint32_t cap, uint32_t npass) {
  UnitLds L;
  L.bterm = reinterpret_cast<uint64_t*>(w);
  L.tl_base = L.bterm + 256;
  L.t_cost = L.tl_base + kTileLds;
  L.tl_trips = reinterpret_cast<uint32_t*>(L.t_cost + cap);
  L.tl_id = L.tl_trips + kTileLds;
  L.t_spec = L.tl_id + kTileLds;
  L.c_info = L.t_spec + cap;
  L.r_off = L.c_info + npass * 256u;
  L.wave_tot = L.r_off + kMaxRanks + 2;
  L.fit = L.wave_tot + 16;
  return L;
}

// Synchronise the T threads that share a unit: one wave needs no s_barrier.
template <int T>
__device__ __forceinline__ void unit_sync() {
  if (T == 64) {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  } else {
    __syncthreads();
  }
}

// fit[dt * 4 + l], bit s: the tensors of subset s (operands 0..3, bit 4 = the fused Spec's
// intermediate) together fit level l when the dtype bits are dt.  Computed by one wave.
__device__ __forceinline__ void build_fit(const DevParams* __restrict__ P, const Shape& S, uint32_t* fit) {
  const uint32_t s = threadIdx.x & 63u;
  for (uint32_t dt = 0; dt < (1u << P->ndt); dt++) {
    uint64_t sum = 0;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if ((uint32_t)i >= P->nops) break;
      const uint32_t bf = P->dt_bit[i] != kNoBit ? (dt >> P->dt_bit[i]) & 1u : P->base_bf16[i];
      sum += (s >> i) & 1u ? S.numel[i] * (bf ? 2u : 4u) : 0;
    }
    sum += (s >> 4) & 1u ? S.numel[4] * 4u : 0;
#pragma unroll
    for (int l = 0; l < 4; l++) {
      const unsigned long long ok = __ballot(s < 32 && sum <= P->cap[l]);
      if (s == 0) fit[dt * 4 + l] = (uint32_t)ok;
    }
  }
}

// Bit v of the result: variant v of the level assignment `info` (DevParams::pos_info) fits.
// f = fit[0..3] in registers serves the common case of no dtype bits.
__device__ __forceinline__ uint32_t admissible_mask(const DevParams* __restrict__ P, const uint32_t* fit,
                                                    const uint32_t f[4], uint32_t info, uint32_t pass) {
  const bool fused = P->kind == kKindF;
  if (P->ndt == 0) {
    uint32_t ok = 1;
#pragma unroll
    for (int l = 0; l < 4; l++) {
      const uint32_t subset = ((info >> (8 + 4 * l)) & 15u) | (fused && pass == (uint32_t)l ? 16u : 0u);
      ok &= (uint32_t)l < P->NL ? f[l] >> subset : 1u;
    }
    return (ok & 1u) ? (1u << P->V) - 1u : 0u;
  }
  const uint32_t ndtpat = 1u << P->ndt;
  uint32_t bits = 0;
  for (uint32_t dt = 0; dt < ndtpat; dt++) {
    uint32_t ok = 1;
#pragma unroll
    for (int l = 0; l < 4; l++) {
      if ((uint32_t)l >= P->NL) break;
      const uint32_t subset = ((info >> (8 + 4 * l)) & 15u) | (fused && pass == (uint32_t)l ? 16u : 0u);
      ok &= fit[dt * 4 + l] >> subset;
    }
    bits |= (ok & 1u) << dt;
  }
  uint32_t mask = 0;
  for (uint32_t lay = 0; lay < (1u << P->nlay); lay++) mask |= bits << (lay * ndtpat);
  return mask;
}

// Move cost per (convert, operand, src, dst, transposed) for this shape: coefficient * elements.
// The coefficients (thread t: entries t, t + T, ... of the 128-entry table, for both conversion
// planes) and the first tile rewrites are fetched at the start of a unit, long before they are needed.
template <int T>
struct Prefetch {
  static constexpr int kCoef = 256 / T < 1 ? 1 : 256 / T;
  uint32_t coef[kCoef];
  TileEntry te;
  uint32_t td;
  bool tvalid;
};

// Tile rewrite e0 + thread of this shape (dims in order, sizes ascending).  With parallel loops
// the same lists of b, m and n follow once more: td = 4 + dim, trips = rounds of `threads` trips.
template <int T>
__device__ __forceinline__ void fetch_tile(const DevParams* __restrict__ P, const Shape& S, uint32_t e0, uint32_t n_tile,
                                           TileEntry& te, uint32_t& td, bool& valid) {
  const uint32_t tid = T == 64 ? (threadIdx.x & 63u) : threadIdx.x;
  const uint32_t e = e0 + tid;
  valid = tid < kTileLds && e < n_tile;
  td = 0;
  te.jt = 0; te.trips = 0;
  if (valid) {
    uint32_t first = 0, q = 0;
#pragma unroll
    for (int a = 0; a < 4; a++) {
      const uint32_t lo = P->tile_off[a][S.si[a]];
      const uint32_t cnt = P->tile_dim_ok[a] ? P->tile_off[a][S.si[a] + 1] - lo : 0u;
      if (e >= first && e < first + cnt) { td = a; q = lo + (e - first); }
      first += cnt;
    }
    if (P->par) {
#pragma unroll
      for (int a = 0; a < 4; a++) {
        if (a == 2) continue;
        const uint32_t lo = P->tile_off[a][S.si[a]];
        const uint32_t cnt = P->tile_off[a][S.si[a] + 1] - lo;
        if (e >= first && e < first + cnt) { td = 4 + a; q = lo + (e - first); }
        first += cnt;
      }
    }
    te = P->tiles[q];
    if (td >= 4) te.trips = (te.trips + P->threads - 1) / P->threads;
  }
}

// Tile rewrites of a shape: the serial loops, and with parallel loops those over b, m, n again.
__device__ __forceinline__ void count_tiles(const DevParams* __restrict__ P, const Shape& S, uint32_t& n_serial,
                                            uint32_t& n_tile) {
  n_serial = 0;
  uint32_t n_par = 0;
#pragma unroll
  for (int d = 0; d < 4; d++) {
    const uint32_t cnt = P->tile_off[d][S.si[d] + 1] - P->tile_off[d][S.si[d]];
    if (P->tile_dim_ok[d]) n_serial += cnt;
    if (P->par && d != 2) n_par += cnt;
  }
  n_tile = n_serial + n_par;
}

// ... into LDS: table offset of the sub-shape's group, trip count, rewrite id.
template <int T>
__device__ __forceinline__ void store_tile(const DevParams* __restrict__ P, const UnitLds& L, const Shape& S, uint32_t shape,
                                           const TileEntry& te, uint32_t d, bool valid) {
  const uint32_t tid = T == 64 ? (threadIdx.x & 63u) : threadIdx.x;
  if (valid) {
    const uint32_t dd = d & 3u;
    const uint32_t j = dd == 0 ? S.si[0] : dd == 1 ? S.si[1] : dd == 2 ? S.si[2] : S.si[3];
    const uint32_t stride = dd == 0 ? P->shape_stride[0] : dd == 1 ? P->shape_stride[1] : dd == 2 ? P->shape_stride[2] : P->shape_stride[3];
    L.tl_base[tid] = (uint64_t)(shape - (j - te.jt) * stride) * P->G;      // the serial table has the same geometry
    L.tl_trips[tid] = te.trips;
    L.tl_id[tid] = (d >= 4 ? P->par_base : P->tile_base) + dd * P->maxs + te.jt;
  }
}

template <int T>
__device__ __forceinline__ void prefetch_unit(const DevParams* __restrict__ P, const Shape& S, uint32_t n_tile, Prefetch<T>& F) {
  const uint32_t tid = T == 64 ? (threadIdx.x & 63u) : threadIdx.x;
#pragma unroll
  for (int i = 0; i < Prefetch<T>::kCoef; i++) {
    const uint32_t e = tid + i * T;
    F.coef[i] = e < 256 ? (&P->mcoef[0][0][0][0])[e & 127u] : 0u;
  }
  fetch_tile<T>(P, S, 0, n_tile, F.te, F.td, F.tvalid);
}

template <int T>
__device__ __forceinline__ void build_move_costs(const DevParams* __restrict__ P, const Shape& S, const Prefetch<T>& F,
                                                 uint64_t* bterm) {
  const uint32_t tid = T == 64 ? (threadIdx.x & 63u) : threadIdx.x;
#pragma unroll
  for (int k = 0; k < Prefetch<T>::kCoef; k++) {
    const uint32_t e = tid + k * T;
    if (e < 256) {
      const uint32_t cv = e >> 7, i = (e >> 5) & 3u, c = F.coef[k];
      const uint64_t n = i == 0 ? S.numel[0] : i == 1 ? S.numel[1] : i == 2 ? S.numel[2] : S.numel[3];
      bterm[e] = c ? mul_or_limit((uint64_t)c + (cv ? P->convert : 0u), n) : 0;   // 0 = the Move does not exist
    }
  }
}

// Tile candidates first, first + step, ... < n_here of the ones staged in LDS, for one task: the
// sub-Spec sits at the same offset `off` inside a smaller shape's group.  trips * sub + s in 96
// bits; reaching 2^62 = overflow.  Candidates from par_from on are parallel loops: their body is
// the serial-only Spec (read from the serial table) and their constant is the synchronisation cost.
__device__ __forceinline__ void task_tiles(const DevParams* __restrict__ P, const UnitLds& L, uint32_t n_here,
                                           uint32_t par_from, uint32_t first, uint32_t step, uint32_t off,
                                           const uint64_t* __restrict__ cost, Eval& e) {
  const uint64_t s_serial = P->s, s_par = P->sync;
  const uint64_t* __restrict__ serial = P->costM;
  for (uint32_t t0 = first; t0 < n_here; t0 += kBatch * step) {
    uint64_t sub[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; u++) {
      const uint32_t t = t0 + u * step;
      sub[u] = kInf;
      if (t < n_here) sub[u] = (t >= par_from ? serial : cost)[L.tl_base[t] + off];     // no request for a candidate that is not there
    }
#pragma unroll
    for (int u = 0; u < kBatch; u++) {
      const uint32_t t = t0 + u * step;
      if (t < n_here) {
        const bool fin = sub[u] != kInf;
        const uint32_t a = L.tl_trips[t];
        const uint64_t lo = (uint64_t)a * (uint32_t)sub[u];
        const uint64_t hi = (uint64_t)a * (uint32_t)(sub[u] >> 32) + (lo >> 32);   // bits 32.. of the product
        const uint64_t c = ((hi << 32) | (uint32_t)lo) + (t >= par_from ? s_par : s_serial);
        const bool over = fin & (((hi >> 30) != 0) | (c >= kLimit));
        e.ovf |= over ? 1u : 0u;
        consider(e, c, L.tl_id[t], fin & !over);
      }
    }
  }
}

// bufferize (FUSED): Matmul into the intermediate, then bias-add+ReLU out of it.  The composition
// of two Matmuls (Section 2.1): the first, (m, k, p), into the intermediate, then the second,
// (m, p, n), out of it; both are entries of the same Matmul table.  The bias-add + ReLU with its
// own bufferize: per level l in which the intermediate fits next to the operands that live there
// (fit: build_fit's words), the bias add into it plus the ReLU out of it.
// Returns the number of candidates evaluated.
__device__ __forceinline__ uint32_t task_bufferize(const DevParams* __restrict__ P, const Shape& S, uint32_t shape,
                                                   uint32_t xpack, uint32_t v, const uint32_t* fit, Eval& e) {
  const uint32_t NL = P->NL, pack = xpack & 0xFFu, pass = xpack >> 8;
  if (P->split) {
    const uint32_t l0 = (pack >> P->pack_shift[0]) & 3u, l1 = (pack >> P->pack_shift[1]) & 3u, l2 = (pack >> P->pack_shift[2]) & 3u;
    const uint32_t y0 = P->lay_bit[0] != kNoBit ? (v >> P->lay_bit[0]) & 1u : 0u;
    const uint32_t y2 = P->lay_bit[2] != kNoBit ? (v >> P->lay_bit[2]) & 1u : 0u;
    const uint64_t sh = (uint64_t)(S.si[1] * P->nsz[3] + S.si[3]);
    const uint32_t va = P->layM[0] != kNoBit ? y0 << P->layM[0] : 0u, vr = P->layE[1] != kNoBit ? y2 << P->layE[1] : 0u;
    uint32_t cnt = 0;
    for (uint32_t l = 0; l < NL; l++) {
      const uint32_t subset = (l0 == l ? 1u : 0u) | (l1 == l ? 2u : 0u) | (l2 == l ? 4u : 0u) | 16u;
      if (!((fit[l] >> subset) & 1u)) continue;
      const uint64_t ca = P->costM[sh * P->GM + ((l0 * NL + l1) * NL + l) * P->VM + va];
      const uint64_t cr = P->costE[sh * P->GE + (l * NL + l2) * P->VE + vr];
      if (ca != kInf && cr != kInf) {
        if (ca + cr >= kLimit) e.ovf = 1; else consider(e, ca + cr, P->buf_id + l);     // each below 2^62: no wrap
      }
      cnt++;
    }
    return cnt;
  }
  const uint32_t l0 = (pack >> P->pack_shift[0]) & 3u, l1 = (pack >> P->pack_shift[1]) & 3u;
  const uint32_t l2 = (pack >> P->pack_shift[2]) & 3u, l3 = (pack >> P->pack_shift[3]) & 3u;
  const uint32_t y0 = P->lay_bit[0] != kNoBit ? (v >> P->lay_bit[0]) & 1u : 0u;
  const uint32_t y1 = P->lay_bit[1] != kNoBit ? (v >> P->lay_bit[1]) & 1u : 0u;
  const uint32_t y3 = P->lay_bit[3] != kNoBit ? (v >> P->lay_bit[3]) & 1u : 0u;
  const uint32_t zc = pass == 0 ? P->zero[0] : pass == 1 ? P->zero[1] : pass == 2 ? P->zero[2] : P->zero[3];
  if (P->chain) {
    const uint32_t y2 = P->lay_bit[2] != kNoBit ? (v >> P->lay_bit[2]) & 1u : 0u;
    const uint32_t x1 = ((l0 * NL + l1) * NL + pass) * P->VM +
                        (P->layM[0] != kNoBit ? y0 << P->layM[0] : 0u) + (P->layM[1] != kNoBit ? y1 << P->layM[1] : 0u);
    const uint32_t x2 = ((pass * NL + l2) * NL + l3) * P->VM +
                        (P->layM[1] != kNoBit ? y2 << P->layM[1] : 0u) + (P->layM[2] != kNoBit ? y3 << P->layM[2] : 0u);
    // the table's k and n lists are this lattice's p list (and k and n lists)
    const uint64_t c1 = P->costM[(uint64_t)((S.si[1] * P->nkM + S.si[2]) * P->nsz[3] + S.si[0]) * P->GM + x1];
    const uint64_t c2 = P->costM[(uint64_t)((S.si[1] * P->nkM + S.si[0]) * P->nsz[3] + S.si[3]) * P->GM + x2];
    if (c1 != kInf && c2 != kInf) {
      const uint64_t z = mul_or_limit(zc, S.numel[4]);
      const uint64_t sum = z + c1;          // each term <= 2^62: no wrap
      if (z >= kLimit || sum >= kLimit || sum + c2 >= kLimit) e.ovf = 1; else consider(e, sum + c2, P->buf_id);
    }
    return 1;
  }
  const uint32_t xm = ((l0 * NL + l1) * NL + pass) * P->VM +
                      (P->layM[0] != kNoBit ? y0 << P->layM[0] : 0u) + (P->layM[1] != kNoBit ? y1 << P->layM[1] : 0u);
  const uint32_t xe = ((pass * NL + l2) * NL + l3) * P->VE + (P->layE[2] != kNoBit ? y3 << P->layE[2] : 0u);
  const uint64_t cm = P->costM[(uint64_t)((S.si[1] * P->nkM + S.si[2] + P->kM_first) * P->nsz[3] + S.si[3]) * P->GM + xm];
  const uint64_t ce = P->costE[(uint64_t)(S.si[1] * P->nszE_n + S.si[3]) * P->GE + xe];
  if (cm != kInf && ce != kInf) {
    const uint64_t z = mul_or_limit(zc, S.numel[4]);
    const uint64_t sum = z + cm;          // each term <= 2^62: no wrap
    if (z >= kLimit || sum >= kLimit || sum + ce >= kLimit) e.ovf = 1; else consider(e, sum + ce, P->buf_id);
  }
  return 1;
}

// The rank loop gives every task a quad of lanes, one per operand: lane `op` of the quad
// evaluates the Moves of operand `op` (to every lower level, same or transposed layout, with or
// without conversion), then the quad's candidates are reduced to the lexicographic minimum of
// (cost, id).  Most ranks of most shapes hold fewer than 16 tasks, so this divides the
// instructions a rank costs (what a small shape's fill is bound by) by about three.
struct MyOperand {
  bool exists;                 // op < number of operands
  bool has_x, can_cv;
  uint32_t sh, xbit, dtbit;    // level field inside the pack; layout / dtype bit of the variant index
  uint32_t id0, brow;          // first Move id of this operand; its row of the Move-cost table
};

__device__ __forceinline__ MyOperand my_operand(const Hot& H, uint32_t op) {
  MyOperand M;
  M.exists = op < H.nops;
  const uint32_t lay = (H.lay_bytes >> (8u * op)) & 0xFFu;
  const uint32_t dt = (H.dt_bytes >> (8u * op)) & 0xFFu;
  M.sh = (H.shift_bytes >> (8u * op)) & 0xFFu;
  M.can_cv = ((H.cv_bits >> op) & 1u) != 0;
  M.has_x = lay != 0xFFu;
  M.xbit = M.has_x ? 1u << (lay & 31u) : 0u;
  M.dtbit = M.can_cv ? 1u << (dt & 31u) : 0u;
  M.id0 = H.move_base + op * (H.NL - 1) * 4u;
  M.brow = op * 32u;
  return M;
}

// One conversion plane (cv) of my operand's Moves: 3 destinations x {same, transposed}.  ci[dst] is
// the (admissible variants | first task) word of the destination's level assignment.  All
// sub-Specs have a lower rank and are final in LDS.
__device__ __forceinline__ void move_plane(const Hot& H, const MyOperand& M, const UnitLds& L, uint32_t q, uint32_t src,
                                           uint32_t v, uint32_t cv, bool on, const uint32_t ci[3], Eval& e,
                                           uint32_t& hi_or) {
  const bool has_dt = H.ndt != 0;
  const uint32_t cvbit = cv ? M.dtbit : 0u;
  const uint32_t brow = cv * 128u + M.brow + src * 8u;
  uint64_t b[6], t[6];
  bool has[6];
#pragma unroll
  for (uint32_t dst = 0; dst < 3; dst++)
#pragma unroll
    for (uint32_t x = 0; x < 2; x++) {
      const uint32_t c = dst * 2 + x, v2 = (v ^ (x ? M.xbit : 0u)) & ~cvbit;
      b[c] = L.bterm[brow + dst * 2u + x];
      has[c] = on && dst < src && (x == 0 || M.has_x) && ((ci[dst] >> v2) & 1u);
      const uint32_t idx = (ci[dst] >> 16) + (has_dt ? __popc(ci[dst] & 0xFFFFu & ((1u << v2) - 1u)) : v2);
      t[c] = L.t_cost[has[c] ? idx : q];
    }
#pragma unroll
  for (uint32_t dst = 0; dst < 3; dst++)
#pragma unroll
    for (uint32_t x = 0; x < 2; x++) {
      const uint32_t c = dst * 2 + x;
      const bool exists = on && dst < src && (x == 0 || M.has_x) && b[c] != 0;     // b == 0: the target has no such Move
      e.n += exists ? 1u : 0u;
      const bool fin = exists & has[c] & (t[c] != kInf);
      const uint64_t cand = t[c] + b[c];                        // t < 2^62 when finite, b <= 2^62: no wrap
      hi_or |= fin ? (uint32_t)(cand >> 32) : 0u;
      consider(e, cand, M.id0 + (dst * 2u + x) * 2u + cv, fin);
    }
}

// Exchange inside a quad of lanes (lane ^ 1, lane ^ 2) without going through LDS.
template <int CTRL>
__device__ __forceinline__ uint32_t quad_swap(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ void quad_min(Eval& e) {
  const uint32_t lo = quad_swap<CTRL>((uint32_t)e.best), hi = quad_swap<CTRL>((uint32_t)(e.best >> 32));
  const uint32_t id = quad_swap<CTRL>(e.arg);
  consider(e, (uint64_t)hi << 32 | lo, id);
}

// One unit = passes [pass0, pass0 + np) of one shape, handled by T threads.
template <int T>
__device__ __forceinline__ void solve_unit(const DevParams* __restrict__ P, const UnitLds& L, uint32_t cap,
                                           const Shape& S, uint32_t shape, uint32_t pass0, uint32_t np,
                                           uint64_t* __restrict__ cost, uint16_t* __restrict__ arg, Eval& tot) {
  const uint32_t tid = T == 64 ? (threadIdx.x & 63u) : threadIdx.x;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t ncombo = P->ncombo;
  const uint64_t group = (uint64_t)shape * P->G;
  const Hot H = load_hot(P);
  uint32_t n_serial, n_tile;
  count_tiles(P, S, n_serial, n_tile);
  Prefetch<T> pre;
  prefetch_unit<T>(P, S, n_tile, pre);

  // ---- 1. admissibility, compaction in rank order (rank-major level assignments, then pass) ----
  constexpr int kIter = 256 / T < 1 ? 1 : 256 / T;   // ncombo <= 256
  uint32_t info[kIter];
#pragma unroll
  for (int it = 0; it < kIter; it++) info[it] = it * T + tid < ncombo ? P->pos_info[it * T + tid] : 0u;
  if (T == 64 || threadIdx.x < 64) build_fit(P, S, L.fit);
  unit_sync<T>();
  uint32_t f[4];
#pragma unroll
  for (int l = 0; l < 4; l++) f[l] = L.fit[l];
  uint32_t n_task = 0;
  if (H.ndt == 0) {
    // No dtype coordinate: the variants of a (level assignment, pass) fit all or none, so a ballot
    // per pass holds everything and the prefix sums are popcounts.  A: level l holds its operands;
    // B: and the intermediate as well.
    const uint32_t V = 1u << H.log2V;
    const bool fused = P->kind == kKindF;
#pragma unroll
    for (int it = 0; it < kIter; it++) {
      if ((uint32_t)(it * T) >= ncombo) break;
      const uint32_t pc = it * T + tid;
      uint32_t A = 0, B = 0;
#pragma unroll
      for (int l = 0; l < 4; l++) {
        const uint32_t sub = (info[it] >> (8 + 4 * l)) & 15u;
        A |= ((uint32_t)l < H.NL ? (f[l] >> sub) & 1u : 1u) << l;
        B |= ((uint32_t)l < H.NL ? (f[l] >> (sub | 16u)) & 1u : 1u) << l;
      }
      bool ok[4];
      unsigned long long bal[4];
      uint32_t before = 0, wave_cnt = 0;
#pragma unroll
      for (int ps = 0; ps < 4; ps++) {
        const uint32_t pass = pass0 + ps;
        ok[ps] = (uint32_t)ps < np && pc < ncombo && (fused ? ((A | 1u << pass) == 15u) && ((B >> pass) & 1u) : A == 15u);
        bal[ps] = __ballot(ok[ps]);
        before += __builtin_amdgcn_mbcnt_hi((uint32_t)(bal[ps] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal[ps], 0u));
        wave_cnt += (uint32_t)__popcll(bal[ps]);
      }
      uint32_t base = n_task + before * V;
      if (T == 64) {
        n_task += wave_cnt * V;
      } else {
        const uint32_t w = threadIdx.x >> 6;
        if (lane == 0) L.wave_tot[w] = wave_cnt * V;
        __syncthreads();
        for (uint32_t i = 0; i < T / 64; i++) {
          const uint32_t t = L.wave_tot[i];
          if (i < w) base += t;
          n_task += t;
        }
        __syncthreads();
      }
      if (pc < ncombo) {
#pragma unroll
        for (int ps = 0; ps < 4; ps++)
          if ((uint32_t)ps < np) {
            const uint32_t xpack = (pass0 + ps) << 8 | (info[it] & 0xFFu);
            if (ps == 0 && (info[it] >> 24)) L.r_off[(info[it] >> 24) - 1u] = base;      // this position opens a rank
            L.c_info[xpack] = (ok[ps] ? (1u << V) - 1u : 0u) | base << 16;
            if (ok[ps]) {
              if (base + V <= cap) {
                if (V >= 4) {
                  for (uint32_t v0 = 0; v0 < V; v0 += 4)
                    *reinterpret_cast<uint4*>(&L.t_spec[base + v0]) =
                        make_uint4(xpack | v0 << 10, xpack | (v0 + 1) << 10, xpack | (v0 + 2) << 10, xpack | (v0 + 3) << 10);
                } else {
                  for (uint32_t v0 = 0; v0 < V; v0++) L.t_spec[base + v0] = xpack | v0 << 10;
                }
              }
              base += V;
            }
          }
      }
    }
  } else {
#pragma unroll
    for (int it = 0; it < kIter; it++) {
      if ((uint32_t)(it * T) >= ncombo) break;
      const uint32_t pc = it * T + tid;
      uint32_t mask[4] = {0, 0, 0, 0}, cnt = 0;
      if (pc < ncombo) {
#pragma unroll
        for (int ps = 0; ps < 4; ps++)
          if ((uint32_t)ps < np) { mask[ps] = admissible_mask(P, L.fit, f, info[it], pass0 + ps); cnt += __popc(mask[ps]); }
      }
      uint32_t incl = cnt;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_up(incl, d, 64);
        if ((int)lane >= d) incl += o;
      }
      uint32_t base = n_task + incl - cnt;
      if (T == 64) {
        n_task += __shfl(incl, 63, 64);
      } else {
        const uint32_t w = threadIdx.x >> 6;
        if (lane == 63) L.wave_tot[w] = incl;
        __syncthreads();
        for (uint32_t i = 0; i < T / 64; i++) {
          const uint32_t t = L.wave_tot[i];
          if (i < w) base += t;
          n_task += t;
        }
        __syncthreads();
      }
      if (pc < ncombo) {
#pragma unroll
        for (int ps = 0; ps < 4; ps++)
          if ((uint32_t)ps < np) {
            const uint32_t xpack = (pass0 + ps) << 8 | (info[it] & 0xFFu);
            if (ps == 0 && (info[it] >> 24)) L.r_off[(info[it] >> 24) - 1u] = base;      // this position opens a rank
            L.c_info[xpack] = mask[ps] | base << 16;
            const uint32_t c = __popc(mask[ps]);
            if (base + c <= cap) {
              uint32_t q = base;
              for (uint32_t m = mask[ps]; m; m &= m - 1) L.t_spec[q++] = xpack | ((uint32_t)__ffs(m) - 1u) << 10;
            }
            base += c;
          }
      }
    }
  }
  if (n_task == 0) return;          // nothing here fits anywhere: the table already says so
  if (n_task > cap) { tot.ovf |= 2u; return; }   // the plan guarantees this cannot happen; reported as an internal error
  if (tid == 0) L.r_off[P->nranks] = n_task;
  build_move_costs<T>(P, S, pre, L.bterm);

  // ---- 3. tile and bufferize candidates of every task (sub-Specs of other shapes / tables: final) ----
  const bool has_buf = P->kind == kKindF || P->split;
  const uint32_t n_per_task = n_tile;          // (the bufferize candidates are counted where they are evaluated)
  for (uint32_t e0 = 0; e0 == 0 || e0 < n_tile; e0 += kTileLds) {
    if (e0) {
      unit_sync<T>();
      fetch_tile<T>(P, S, e0, n_tile, pre.te, pre.td, pre.tvalid);
    }
    store_tile<T>(P, L, S, shape, pre.te, pre.td, pre.tvalid);
    unit_sync<T>();
    const uint32_t n_here = n_tile - e0 < kTileLds ? n_tile - e0 : kTileLds;
    const uint32_t par_from = n_serial > e0 ? (n_serial - e0 < n_here ? n_serial - e0 : n_here) : 0u;
    if (n_task * 2 <= T) {
      // few tasks: a quad of lanes per task, every fourth candidate each (fewer reads one after the other)
      for (uint32_t qb = 0; qb < n_task; qb += T / 4) {
        const bool active = qb + (tid >> 2) < n_task;
        const uint32_t q = active ? qb + (tid >> 2) : 0u, sub4 = tid & 3u;
        const uint32_t sp = L.t_spec[q];
        const uint32_t xpack = sp & 0x3FFu, v = (sp >> 10) & 31u;
        Eval e;
        e.ovf = 0; e.best = kInf; e.arg = kNone;
        if (sub4 == 0) {
          if (e0 == 0) { if (has_buf) { const uint32_t nb = task_bufferize(P, S, shape, xpack, v, L.fit, e); tot.n += active ? nb : 0u; } }
          else { e.best = L.t_cost[q]; e.arg = sp >> 16; }
        }
        task_tiles(P, L, n_here, par_from, sub4, 4, entry_offset(H, xpack, v), cost, e);
        if (active) tot.ovf |= e.ovf;
        quad_min<0xB1>(e);
        quad_min<0x4E>(e);
        if (active && sub4 == 0) {
          L.t_cost[q] = e.best;
          L.t_spec[q] = (sp & 0xFFFFu) | e.arg << 16;
        }
      }
    } else {
      for (uint32_t q = tid; q < n_task; q += T) {
        const uint32_t sp = L.t_spec[q];
        const uint32_t xpack = sp & 0x3FFu, v = (sp >> 10) & 31u;
        Eval e;
        e.ovf = 0;
        if (e0 == 0) {
          e.best = kInf; e.arg = kNone;
          if (has_buf) tot.n += task_bufferize(P, S, shape, xpack, v, L.fit, e);
        } else {
          e.best = L.t_cost[q]; e.arg = sp >> 16;
        }
        task_tiles(P, L, n_here, par_from, 0, 1, entry_offset(H, xpack, v), cost, e);
        L.t_cost[q] = e.best;
        L.t_spec[q] = (sp & 0xFFFFu) | e.arg << 16;
        tot.ovf |= e.ovf;
      }
    }
  }
  tot.n += n_per_task * ((n_task > tid ? n_task - tid + T - 1 : 0u) / T);
  unit_sync<T>();

  // microkernels whose shape predicate holds for this shape (uniform)
  uint32_t mk_shape = 0;
  for (uint32_t j = 0; j < P->nmk; j++) mk_shape |= (mk_shape_reps(P, S, j) ? 1u : 0u) << j;

  // ---- 4. rank by rank: microkernels and Moves, then the parked tile/bufferize candidate ----
  const uint32_t op = tid & 3u;
  const MyOperand M = my_operand(H, op);
  for (uint32_t r = 0; r < P->nranks; r++) {
    const uint32_t t0 = L.r_off[r], t1 = L.r_off[r + 1];
    if (t0 == t1) continue;
    for (uint32_t qb = t0; qb < t1; qb += T / 4) {
      const bool active = qb + (tid >> 2) < t1;
      const uint32_t q = active ? qb + (tid >> 2) : t0;        // idle lanes read task t0 and drop the result
      const uint32_t sp = L.t_spec[q];
      const uint32_t xpack = sp & 0x3FFu, v = (sp >> 10) & 31u;
      // my operand's Moves
      Eval e;
      e.best = kInf; e.arg = kNone; e.n = 0; e.ovf = 0;
      uint32_t hi_or = 0;           // OR of the high words of all finite Move candidates
      const uint32_t src = (xpack >> M.sh) & 3u;
      const bool on = active && M.exists && src != 0;
      if (__any(on)) {
        uint32_t ci[3];
#pragma unroll
        for (uint32_t dst = 0; dst < 3; dst++) ci[dst] = L.c_info[on && dst < src ? xpack - ((src - dst) << M.sh) : xpack];
        move_plane(H, M, L, q, src, v, 0, on, ci, e, hi_or);
        const bool cv_on = on && M.can_cv && (v & M.dtbit);
        if (__any(cv_on)) move_plane(H, M, L, q, src, v, 1, cv_on, ci, e, hi_or);
      }
      if (hi_or >> 30) e.ovf = 1;   // bit 62 of some finite candidate: the solve reports overflow
      tot.n += e.n;
      tot.ovf |= e.ovf;
      quad_min<0xB1>(e);            // lanes ^ 1
      quad_min<0x4E>(e);            // lanes ^ 2
      if (active && op == 0) {
        // the quad's first lane adds the microkernels (lowest ids) and the parked candidate, and stores
        Eval f;
        f.best = L.t_cost[q]; f.arg = sp >> 16; f.n = 0; f.ovf = 0;
        consider(f, e.best, e.arg);
        if (mk_shape) {
          for (uint32_t mm = P->mk_entry[(xpack & 0xFFu) * P->V + v] & mk_shape; mm; mm &= mm - 1) {
            const uint32_t j = (uint32_t)__ffs(mm) - 1u;
            const uint64_t k = mul_or_limit(P->mk_cost[j], mk_shape_reps(P, S, j));
            if (k >= kLimit) f.ovf = 1; else consider(f, k, j);
            f.n++;
          }
        }
        L.t_cost[q] = f.best;
        L.t_spec[q] = (sp & 0xFFFFu) | f.arg << 16;
        tot.n += f.n;
        tot.ovf |= f.ovf;
      }
    }
    unit_sync<T>();
  }
  // Results to the table after the last rank, a task per lane: inside the rank loop every chunk
  // would wait for the previous chunk's stores (stores count on the same counter as loads here).
  for (uint32_t q = tid; q < n_task; q += T) {
    const uint32_t sp = L.t_spec[q];
    const uint32_t off = entry_offset(H, sp & 0x3FFu, (sp >> 10) & 31u);
    cost[group + off] = L.t_cost[q];
    arg[group + off] = (uint16_t)(sp >> 16);
  }
}

__device__ __forceinline__ void flush_counters(Counters* __restrict__ ctr, const Eval& tot) {
  uint32_t n_rw = tot.n;
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) n_rw += __shfl_down(n_rw, d, 64);
  if ((threadIdx.x & 63u) == 0 && n_rw) atomicAdd(&ctr->n_rewrites[blockIdx.x % kCtrSlots], (unsigned long long)n_rw);
  if (tot.ovf) atomicOr(&ctr->overflow, tot.ovf);
}

// Plan: one wave per kPlanShapes consecutive shapes (the per-assignment table and the parameters
// stay in registers across them).  Counts the entries that fit per passive-level slice, marks them
// in a bit map in table order (bit = cell; read by the compression pass) and classifies the shape:
// bit 8 = one LDS slice holds it whole (bit 9: even a wave's small slice); else bits 0..3 = passive-level
// slices that fit an LDS slice, bits 4..7 = slices that need the large one.  sort_work_kernel turns the classes into per-level work lists.
constexpr uint32_t kPlanShapes = 8;

__global__ __launch_bounds__(256) void plan_kernel(const DevParams* __restrict__ P, uint32_t n_shapes,
                                                   uint32_t cap_whole, uint32_t cap_slice, uint32_t cap_wave,
                                                   uint32_t* __restrict__ shape_class, uint32_t* __restrict__ fitmap,
                                                   Counters* __restrict__ ctr, uint4* __restrict__ cost16,
                                                   uint4* __restrict__ arg16) {
  __shared__ uint32_t fit_all[4][16];
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
  uint32_t* fit = fit_all[wave];
  const uint32_t npass = P->npass, ncombo = P->ncombo, V = P->V, nb = npass * V;
  const Hot H = load_hot(P);
  uint32_t info[4], off0[4];
#pragma unroll
  for (int it = 0; it < 4; it++) {
    info[it] = it * 64 + lane < ncombo ? P->pos_info[it * 64 + lane] : 0u;
    off0[it] = entry_offset(H, info[it] & 0xFFu, 0);      // pass 0, variant 0 of this level assignment
  }
  unsigned long long n_adm = 0;
  const uint32_t first_shape = (blockIdx.x * 4 + wave) * kPlanShapes;
  for (uint32_t shape = first_shape; shape < first_shape + kPlanShapes && shape < n_shapes; shape++) {
    if (cost16) {
      // (INF, NONE) = all-ones over the shape's whole group: the level kernels overwrite what fits
      const uint4 ones = make_uint4(~0u, ~0u, ~0u, ~0u);
      const uint32_t nc = P->G >> 1, na = P->G >> 3;       // 16-byte pieces (G is a multiple of 8)
      uint4* c16 = cost16 + (size_t)shape * nc;
      uint4* a16 = arg16 + (size_t)shape * na;
      for (uint32_t i = lane; i < nc; i += 64) c16[i] = ones;
      for (uint32_t i = lane; i < na; i += 64) a16[i] = ones;
    }
    Shape S;
    load_shape(P, shape, S);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    build_fit(P, S, fit);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    uint32_t f[4];
#pragma unroll
    for (int l = 0; l < 4; l++) f[l] = fit[l];
    const uint64_t group = (uint64_t)shape * P->G;
    uint32_t cnt[4] = {0, 0, 0, 0};
#pragma unroll
    for (int it = 0; it < 4; it++) {
      if ((uint32_t)(it * 64) >= ncombo) break;
      if (it * 64 + lane >= ncombo) continue;
      unsigned long long bits = 0;
#pragma unroll
      for (int ps = 0; ps < 4; ps++)
        if ((uint32_t)ps < npass) {
          const uint32_t m = admissible_mask(P, fit, f, info[it], ps);
          cnt[ps] += __popc(m);
          bits |= (unsigned long long)m << (ps * V);
        }
      if (nb == 32 || nb == 64) {
        // whole words of the map (the group size is a multiple of nb): stored, the map is not zeroed
        uint32_t* w = fitmap + ((group + off0[it]) >> 5);
        w[0] = (uint32_t)bits;
        if (nb == 64) w[1] = (uint32_t)(bits >> 32);
      } else if (bits) {
        const uint64_t cell0 = group + off0[it];
        const uint32_t sh = (uint32_t)(cell0 & 31u);
        uint32_t* w = fitmap + (cell0 >> 5);
        atomicOr(w, (uint32_t)(bits << sh));
        if (sh + nb > 32) {
          atomicOr(w + 1, (uint32_t)(bits >> (32 - sh)));
          if (sh + nb > 64) atomicOr(w + 2, (uint32_t)(bits >> (64 - sh)));
        }
      }
    }
    uint32_t total = 0;
#pragma unroll
    for (int ps = 0; ps < 4; ps++) {
#pragma unroll
      for (int d = 32; d > 0; d >>= 1) cnt[ps] += __shfl_down(cnt[ps], d, 64);
      cnt[ps] = __shfl(cnt[ps], 0, 64);
      total += cnt[ps];
    }
    if (lane == 0) {
      n_adm += total;
      uint32_t cls = 0;
      if (total && total <= cap_whole) cls = total <= cap_wave ? 0x300u : 0x100u;
      else
        for (uint32_t ps = 0; ps < npass; ps++)
          if (cnt[ps]) cls |= 1u << (cnt[ps] <= cap_slice ? ps : 4 + ps);
      shape_class[shape] = cls;
    }
  }
  if (lane == 0 && n_adm) atomicAdd(&ctr->n_admissible[blockIdx.x % kCtrSlots], n_adm);
}

// One workgroup per dependency level: walks the level's shapes in index order and writes its work
// lists and their lengths: whole shapes (the small ones from the front of the level's stretch of
// list_whole, the others from its back), slices, and wide slices.
constexpr uint32_t kSortThreads = 1024;
__global__ __launch_bounds__(kSortThreads) void sort_work_kernel(const uint32_t* __restrict__ level_shapes,
                                                                 const uint32_t* __restrict__ level_off, uint32_t n_levels,
                                                                 uint32_t npass, const uint32_t* __restrict__ shape_class,
                                                                 uint32_t* __restrict__ list_whole, uint32_t* __restrict__ list_slice,
                                                                 uint32_t* __restrict__ list_wide, uint32_t* __restrict__ list_cnt) {
  constexpr uint32_t kWaves = kSortThreads / 64;
  __shared__ unsigned long long wave_sum[kWaves];
  __shared__ uint32_t run[4];
  const uint32_t lv = blockIdx.x, first = level_off[lv], n = level_off[lv + 1] - first;
  if (threadIdx.x < 4) run[threadIdx.x] = 0;
  __syncthreads();
  for (uint32_t base = 0; base < n; base += kSortThreads) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t shape = i < n ? level_shapes[first + i] : 0u;
    const uint32_t cls = i < n ? shape_class[shape] : 0u;
    const uint32_t cw = (cls >> 9) & 1u, cb = ((cls >> 8) & 1u) & ~cw, cs = __popc(cls & 15u), cx = __popc((cls >> 4) & 15u);
    // four counts in 16-bit fields (per kSortThreads threads: <= 1024, 4096, 4096, 1024)
    const unsigned long long packed = (unsigned long long)cw | (unsigned long long)cs << 16 | (unsigned long long)cx << 32 |
                                      (unsigned long long)cb << 48;
    unsigned long long incl = packed;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const unsigned long long o = __shfl_up(incl, d, 64);
      if ((int)(threadIdx.x & 63u) >= d) incl += o;
    }
    if ((threadIdx.x & 63u) == 63) wave_sum[threadIdx.x >> 6] = incl;
    __syncthreads();
    unsigned long long excl = incl - packed, tot = 0;
    for (uint32_t w = 0; w < kWaves; w++) {
      if (w < (threadIdx.x >> 6)) excl += wave_sum[w];
      tot += wave_sum[w];
    }
    uint32_t ow = run[0] + (uint32_t)(excl & 0xFFFFu), os = run[1] + (uint32_t)((excl >> 16) & 0xFFFFu);
    uint32_t ox = run[2] + (uint32_t)((excl >> 32) & 0xFFFFu);
    if (cw) list_whole[first + ow] = shape;
    if (cb) list_whole[first + n - 1u - (run[3] + (uint32_t)(excl >> 48))] = shape;
    for (uint32_t ps = 0; ps < npass; ps++) {
      if ((cls >> ps) & 1u) list_slice[(size_t)first * npass + os++] = shape * npass + ps;
      if ((cls >> (4 + ps)) & 1u) list_wide[(size_t)first * npass + ox++] = shape * npass + ps;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      run[0] += (uint32_t)(tot & 0xFFFFu); run[1] += (uint32_t)((tot >> 16) & 0xFFFFu);
      run[2] += (uint32_t)((tot >> 32) & 0xFFFFu); run[3] += (uint32_t)(tot >> 48);
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    list_cnt[lv] = run[0]; list_cnt[n_levels + lv] = run[1]; list_cnt[2 * n_levels + lv] = run[2];
    list_cnt[3 * n_levels + lv] = run[3];
  }
}

// One dependency level, the items an LDS slice holds: first the larger ones
// (whole shapes from the back of the level's stretch of list_whole, then slices), which take
// longest, then the small whole shapes, which fill the gaps at the end.  T threads per item: one
// wave when the level has enough items to fill the chip, four when it has few (then an item's
// tasks are spread over more lanes).
template <int T>
__global__ __launch_bounds__(T) __attribute__((amdgpu_waves_per_eu(1, 4))) void fill_kernel(
    const DevParams* __restrict__ P, const uint32_t* __restrict__ list_whole, uint32_t n_stretch, uint32_t n_bigwhole,
    const uint32_t* __restrict__ list_slice, uint32_t n_slice, uint32_t cap, uint64_t* __restrict__ cost,
    uint16_t* __restrict__ arg, Counters* __restrict__ ctr) {
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t n_big = n_bigwhole + n_slice;
  uint32_t shape, pass0 = 0, np = P->npass;
  if (blockIdx.x < n_bigwhole) {
    shape = list_whole[n_stretch - 1u - blockIdx.x];
  } else if (blockIdx.x < n_big) {
    const uint32_t unit = list_slice[blockIdx.x - n_bigwhole];
    shape = unit / P->npass; pass0 = unit - shape * P->npass; np = 1;
  } else {
    shape = list_whole[blockIdx.x - n_big];
  }
  Shape S;
  load_shape(P, shape, S);
  const UnitLds L = carve(smem, cap, P->npass);
  Eval tot;
  tot.n = 0; tot.ovf = 0;
  solve_unit<T>(P, L, cap, S, shape, pass0, np, cost, arg, tot);
  flush_counters(ctr, tot);
}

// The slices too large for a wave's LDS slice: one workgroup of TB threads each (kBigBlock, or
// twice as many on levels with so few of them that most compute units would hold one or none).
template <int TB>
__global__ __launch_bounds__(TB) __attribute__((amdgpu_waves_per_eu(1, 4))) void fill_big_kernel(const DevParams* __restrict__ P,
                                                             const uint32_t* __restrict__ list_wide, uint32_t cap,
                                                             uint64_t* __restrict__ cost, uint16_t* __restrict__ arg,
                                                             Counters* __restrict__ ctr) {
  extern __shared__ __align__(16) unsigned char smem[];
  const UnitLds L = carve(smem, cap, P->npass);
  Eval tot;
  tot.n = 0; tot.ovf = 0;
  const uint32_t unit = list_wide[blockIdx.x];
  const uint32_t shape = unit / P->npass, pass = unit % P->npass;
  Shape S;
  load_shape(P, shape, S);
  solve_unit<TB>(P, L, cap, S, shape, pass, 1, cost, arg, tot);
  flush_counters(ctr, tot);
}

// (INF, NONE) are all-ones bytes: stream 16 bytes per lane and store over both tables.
__global__ __launch_bounds__(256) void fill_ones_kernel(uint4* __restrict__ p, size_t n16) {
  const uint4 ones = make_uint4(~0u, ~0u, ~0u, ~0u);
  for (size_t i = (size_t)blockIdx.x * 256u + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256u) p[i] = ones;
}

// The same in workgroups that end after 16 KB each: beside the latency-bound kernels of another
// stream the compute units' wave slots then turn over all the time, and those kernels' workgroups
// are placed as soon as they are launched (a grid of workgroups that live as long as the whole
// stream of stores holds every slot until it ends).
__global__ __launch_bounds__(256) void fill_ones_short_kernel(uint4* __restrict__ p, size_t n16) {
  const uint4 ones = make_uint4(~0u, ~0u, ~0u, ~0u);
  const size_t i0 = (size_t)blockIdx.x * 1024u + threadIdx.x;
#pragma unroll
  for (int k = 0; k < 4; k++) {
    const size_t i = i0 + (size_t)k * 256u;
    if (i < n16) p[i] = ones;
  }
}

void launch_fill_ones(void* p, size_t bytes, hipStream_t stream, bool short_lived) {
  const size_t n16 = bytes / 16;
  if (n16 && short_lived) {
    size_t done = 0;
    while (done < n16) {          // (grids stay below 2^31 workgroups)
      const size_t part = n16 - done < ((size_t)1 << 40) ? n16 - done : ((size_t)1 << 40);
      hipLaunchKernelGGL(fill_ones_short_kernel, dim3((uint32_t)((part + 1023) / 1024)), dim3(256), 0, stream, (uint4*)p + done, part);
      done += part;
    }
  } else if (n16) {
    const size_t blocks = (n16 + 255) / 256;
    hipLaunchKernelGGL(fill_ones_kernel, dim3((uint32_t)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, stream,
                       (uint4*)p, n16);
  }
  if (bytes % 16) (void)hipMemsetAsync((char*)p + n16 * 16, 0xFF, bytes % 16, stream);
}

// Tasks per LDS slice: a whole shape's group when it has at most kSmallCap entries, else
// kSlicedCap (a smaller slice, i.e. more items in flight per CU, pays once shapes are split into
// passive-level slices anyway: measured 256 < 320 < 192 < 512 < 128 on the fused lattice).
uint32_t fill_wave_cap(uint32_t G) { return G <= kSmallCap ? G : kSlicedCap; }

// ---------------------------------------------------------------- memory bounds as coordinates
// Sections 2.2 and 2.4.4: a Spec carries, per level of finite capacity, the bytes an implementation
// may still allocate there; a Move allocates the moved operand's buffer in its destination, so it
// needs that many bytes of the destination's bound and leaves its body the rest, rounded down to
// a power of two (or zero).  There is no admissibility test: the bounds decide.
//
// A Move lowers the sum of the operand levels (the rank) within a shape, and a tile goes to the
// same level assignment of a smaller shape (a lower dependency level of shapes), so the Specs of
// (level l, rank r) depend only on (l, r' < r) and (l' < l, r): all pairs on one diagonal
// l + r = d are independent, and one launch takes a whole diagonal, one segment of workgroups per
// pair.  One lane per Spec, every candidate a gather from finished entries.  Lane -> (shape of
// the level, level assignment of the rank, level of the fused Spec's intermediate, bound vector,
// variant), variant fastest.  A bufferize (fused Spec) allocates the intermediate in its level:
// it needs 4 * m * n bytes of that level's bound, and both stages get the rest, rounded down.
//
// The same kernel fills two further kinds of lattice, which also are gathers from finished
// entries.  Move Specs (Section 2.2; kind kKindV): two tensors, no Move rewrites; where a bounded
// lattice has its bounds they have the abstract values of Section 2.4.3 (contiguousness and
// aligned flag of source and destination), which a tile changes and the vector-move microkernels
// test.  And the Matmul whose Moves are Move Specs (Section 2, Memory Movement; Section 3): the
// plain Matmul Specs with their admissibility test, where a Move costs m(src) + m(dest) in cache
// lines plus the load and store Move Specs, read from the Move table.
__device__ __forceinline__ uint64_t add_or_limit(uint64_t a, uint64_t b) {
  return (a >= kLimit || b >= kLimit || a + b >= kLimit) ? kLimit : a + b;
}

// MODE 0: memory bounds as coordinates; 1: Move Specs; 2: the Matmul whose Moves are Move Specs.
template <int MODE>
__global__ __launch_bounds__(256) void fill_bounded_kernel(const DevParams* __restrict__ P,
                                                           const uint32_t* __restrict__ all_level_shapes, const BoundSegs segs,
                                                           uint64_t* cost, uint16_t* __restrict__ arg,
                                                           Counters* __restrict__ ctr) {
  __shared__ uint32_t wave_n[4], wave_adm[4];
  uint32_t seg = 0;
  while (seg + 1 < segs.n && blockIdx.x >= segs.block0[seg + 1]) seg++;
  const uint32_t rank = segs.rank[seg], n_level_shapes = segs.n_shapes[seg];
  const uint32_t* __restrict__ level_shapes = all_level_shapes + segs.first_shape[seg];
  const uint32_t V = P->V, Q = P->Q, npass = P->npass, nops = P->nops;
  const uint32_t c0 = P->rank_off[rank], ncr = P->rank_off[rank + 1] - c0;
  const uint64_t per_shape = (uint64_t)ncr * npass * Q * V;
  const uint64_t t = (uint64_t)(blockIdx.x - segs.block0[seg]) * 256u + threadIdx.x;
  const bool active = t < per_shape * n_level_shapes;
  Eval e;
  e.best = kInf; e.arg = kNone; e.n = 0; e.ovf = 0;
  uint32_t n_adm = 0;
  if (active) {
    // (an active lane's index is below the number of Specs of the lattice, which fits 32 bits)
    const uint32_t sl = (uint32_t)t / (uint32_t)per_shape;
    uint32_t r = (uint32_t)t - sl * (uint32_t)per_shape;
    const uint32_t ci = r / (npass * Q * V);
    r -= ci * npass * Q * V;
    const uint32_t pass = r / (Q * V);
    r -= pass * Q * V;
    const uint32_t q = r / V, v = r - q * V;
    const uint32_t shape = level_shapes[sl];
    Shape S;
    load_shape(P, shape, S);
    const uint32_t pack = P->pos_info[c0 + ci] & 0xFFu;
    uint32_t lv[4] = {0, 0, 0, 0}, combo = 0;
#pragma unroll
    for (int i = 0; i < 4; i++)
      if ((uint32_t)i < nops) { lv[i] = (pack >> P->pack_shift[i]) & 3u; combo += lv[i] * P->lvpow[i]; }
    uint32_t qi[4] = {0, 0, 0, 0};
    {
      uint32_t rem = q;
#pragma unroll
      for (int a = 0; a < 4; a++)
        if ((uint32_t)a < P->nlim) { qi[a] = rem / P->lim_stride[a]; rem -= qi[a] * P->lim_stride[a]; }
    }
    const uint64_t group = (uint64_t)shape * P->G;
    const uint32_t off = ((combo * npass + pass) * Q + q) * V + v;
    constexpr bool move_specs = MODE == 1, moves = MODE == 2;

    // Where Moves are Specs the lattice is the plain Matmul's: a Spec whose operands do not fit
    // their levels has no implementation and evaluates nothing.
    bool admissible = true;
    const auto layout_of = [&](int i) { return P->lay_bit[i] != kNoBit ? (v >> P->lay_bit[i]) & ((1u << P->lay_w[i]) - 1u) : 0u; };
    if (move_specs) {
      // no such tensor: a packed layout with a broken strip, more adjacent dimensions than the tensor can have
      if (P->xw == 4) {
#pragma unroll
        for (int ts = 0; ts < 2; ts++) {
          const uint32_t y = layout_of(ts);
          admissible = admissible && layout_fits(y, (uint32_t)S.d[3], P->strip) && qi[2 * ts] <= max_contig(y, (uint32_t)S.d[3], P->strip);
        }
      }
      n_adm = admissible ? 1u : 0u;
    }
    if (moves) {
      if (P->xw == 4) {
#pragma unroll
        for (int i = 0; i < 3; i++) {
          const uint32_t cols = (uint32_t)(i == 0 ? S.d[2] : S.d[3]);
          admissible = admissible && (layout_of(i) < 2 || cols % P->strip == 0);      // whole tensors: whole strips
        }
      }
#pragma unroll
      for (int l = 0; l < 4; l++) {
        uint64_t bytes = 0;
#pragma unroll
        for (int i = 0; i < 3; i++) {
          const uint32_t bf = P->dt_bit[i] != kNoBit ? (v >> P->dt_bit[i]) & 1u : P->base_bf16[i];
          bytes += lv[i] == (uint32_t)l ? S.numel[i] * (bf ? 2u : 4u) : 0u;
        }
        admissible = admissible && ((uint32_t)l >= P->NL || bytes <= P->cap[l]);
      }
      n_adm = admissible ? 1u : 0u;
    }
    if (admissible) {

    // microkernels
    const uint32_t mm = P->mk_entry[pack * V + v];
    for (uint32_t j = 0; j < P->nmk; j++) {
      if (!((mm >> j) & 1u)) continue;
      const uint64_t reps = mk_shape_reps(P, S, j);
      if (!reps) continue;
      if (move_specs && P->mk_kind[j] >= 6u) {
        // vector moves: the inner dimension of both tensors adjacent in memory; the aligned form: both aligned
        if (qi[0] < 1u || qi[2] < 1u) continue;
        if (P->mk_kind[j] == 7u && !(qi[1] && qi[3])) continue;
        // a row of whole strips: the strips must be whole vectors
        if (P->xw == 4 && S.d[3] >= P->strip && P->strip % P->mk_lanes[j] != 0 && (layout_of(0) >= 2 || layout_of(1) >= 2)) continue;
      }
      const uint64_t k = mul_or_limit(P->mk_cost[j], reps);
      if (k >= kLimit) e.ovf = 1; else consider(e, k, j);
      e.n++;
    }

    // Moves (a Move Spec has none)
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if ((uint32_t)i >= nops || move_specs) continue;
      const uint32_t src = lv[i];
      const bool has_dt = P->dt_bit[i] != kNoBit, has_lay = P->lay_bit[i] != kNoBit;
      const uint32_t bf = has_dt ? (v >> P->dt_bit[i]) & 1u : P->base_bf16[i];
      const uint64_t numel = S.numel[i];
      // cache lines of the operand as f32 and as bf16 (Section 3, m(t)), once per operand
      uint64_t lines_f32 = 0, lines_bf16 = 0;
      if (moves) {
        const uint64_t line = P->line_bytes;
        if (P->line_mask || line == 1) {
          const uint32_t sh = 31u - (uint32_t)__clz((int)P->line_bytes);
          lines_f32 = (numel * 4u + line - 1) >> sh; lines_bf16 = (numel * 2u + line - 1) >> sh;
        } else {
          lines_f32 = (numel * 4u + line - 1) / line; lines_bf16 = (numel * 2u + line - 1) / line;
        }
      }
      for (uint32_t dst = 0; dst < src; dst++)
        for (uint32_t x = 0; x < (moves ? P->xw : 2u); x++)          // the Move leaves the operand in layout (its own) xor x
          for (uint32_t cv = 0; cv < 2; cv++) {
            if (x && !has_lay) continue;
            if (x >= 2 && P->lay_w[i] != 2) continue;
            if (cv && !(P->can_convert[i] && has_dt && bf)) continue;
            const uint32_t child_bf = cv ? 0u : bf;
            if (moves) {
              // the alloc-binding: m(src) + m(dest), the load Move Spec (operands that are read), the
              // body, the store Move Spec (operands that are written); the operand is rows x cols
              const uint32_t ri = i == 1 ? S.si[2] : S.si[1], ci = i == 0 ? S.si[2] : S.si[3];
              const uint64_t groupV = (uint64_t)(ri * P->nszV + ci) * P->GV;
              const uint32_t y0 = layout_of(i), y1 = y0 ^ x;
              // both tensors fresh: every physical dimension adjacent, aligned
              const uint32_t top0 = y0 >= 2 ? 3u : 2u, top1 = y1 >= 2 ? 3u : 2u;
              const uint32_t q_load = top0 * P->limV_stride[0] + P->limV_stride[1] + top1 * P->limV_stride[2] + P->limV_stride[3];
              const uint32_t q_store = top1 * P->limV_stride[0] + P->limV_stride[1] + top0 * P->limV_stride[2] + P->limV_stride[3];
              auto variantV = [&](uint32_t ys, uint32_t yd, uint32_t fs, uint32_t fd) {
                return (P->layV[0] != kNoBit ? ys << P->layV[0] : 0u) + (P->layV[1] != kNoBit ? yd << P->layV[1] : 0u) +
                       (P->dtV[0] != kNoBit ? fs << P->dtV[0] : 0u) + (P->dtV[1] != kNoBit ? fd << P->dtV[1] : 0u);
              };
              uint64_t c_load = 0, c_store = 0;
              if (P->access[i] != kWrite)
                c_load = P->costM[groupV + ((src * P->NL + dst) * P->QV + q_load) * P->VV + variantV(y0, y1, bf, child_bf)];
              if (P->access[i] != kRead)
                c_store = P->costM[groupV + ((dst * P->NL + src) * P->QV + q_store) * P->VV + variantV(y1, y0, child_bf, bf)];
              const uint32_t combo_c = combo - (src - dst) * P->lvpow[i];
              uint32_t v_c = v ^ (x ? x << P->lay_bit[i] : 0u);
              if (cv) v_c &= ~(1u << P->dt_bit[i]);
              const uint64_t sub = cost[group + (uint64_t)((combo_c * npass + pass) * Q + q) * V + v_c];
              const uint64_t lines_s = bf ? lines_bf16 : lines_f32, lines_d = child_bf ? lines_bf16 : lines_f32;
              const uint32_t ws = src == 1 ? P->weight[1] : src == 2 ? P->weight[2] : P->weight[3];
              const uint32_t wd = dst == 0 ? P->weight[0] : dst == 1 ? P->weight[1] : P->weight[2];
              const uint32_t id = P->move_base + (((uint32_t)i * (P->NL - 1u) + dst) * P->xw + x) * 2u + cv;
              if (sub != kInf && c_load != kInf && c_store != kInf) {
                uint64_t tot = add_or_limit(mul_or_limit(lines_s, ws), mul_or_limit(lines_d, wd));
                tot = add_or_limit(add_or_limit(tot, c_load), add_or_limit(c_store, sub));
                if (tot >= kLimit) e.ovf = 1; else consider(e, tot, id);
              }
              e.n++;
              continue;
            }
            const uint32_t coef = P->mcoef[i][src][dst][x];
            if (!coef) continue;
            uint32_t qc = q;
            const uint32_t la = P->lim_of_level[dst];
            if (la != kNoBit) {
              const uint32_t qa = la == 0 ? qi[0] : la == 1 ? qi[1] : la == 2 ? qi[2] : qi[3];
              const uint64_t bytes = numel * (child_bf ? 2u : 4u);
              const uint64_t have = qa ? 1ull << (qa - 1u) : 0ull;
              if (bytes > have) continue;                       // the buffer does not fit the bound: no such rewrite
              const uint64_t left = have - bytes;
              const uint32_t qn = left ? 64u - (uint32_t)__clzll((long long)left) : 0u;
              qc = q - (qa - qn) * P->lim_stride[la];
            }
            const uint32_t combo_c = combo - (src - dst) * P->lvpow[i];
            uint32_t v_c = v ^ (x ? 1u << P->lay_bit[i] : 0u);
            if (cv) v_c &= ~(1u << P->dt_bit[i]);
            const uint64_t sub = cost[group + (uint64_t)((combo_c * npass + pass) * Q + qc) * V + v_c];
            const uint64_t b = mul_or_limit((uint64_t)coef + (cv ? P->convert : 0u), numel);
            const uint32_t id = P->move_base + (((uint32_t)i * (P->NL - 1u) + dst) * 2u + x) * 2u + cv;
            if (sub != kInf) {
              if (b >= kLimit || sub + b >= kLimit) e.ovf = 1; else consider(e, sub + b, id);
            }
            e.n++;
          }
    }

    // tiles: the same entry of a smaller shape's group
    const uint64_t s = P->s;
#pragma unroll
    for (int d = 0; d < 4; d++) {
      if (!P->tile_dim_ok[d]) continue;
      for (uint32_t te_i = P->tile_off[d][S.si[d]]; te_i < P->tile_off[d][S.si[d] + 1]; te_i++) {
        const TileEntry te = P->tiles[te_i];
        const uint32_t child = shape - (S.si[d] - te.jt) * P->shape_stride[d];
        uint32_t off_c = off;
        if (move_specs) {
          // Section 2.4.3: what is known of a tile of either tensor.  Cutting the inner dimension
          // leaves only that dimension adjacent; the tile is aligned only if the tensor was aligned
          // and contiguous and the tile's rows (and so the tile) are whole cache lines.
          const uint32_t r2 = d == 1 ? P->sizes[1][te.jt] : (uint32_t)S.d[1], c2 = d == 3 ? P->sizes[3][te.jt] : (uint32_t)S.d[3];
          const uint32_t strip = P->strip ? P->strip : 1u;
          uint32_t qc = 0;
#pragma unroll
          for (int ts = 0; ts < 2; ts++) {
            const uint32_t y = layout_of(ts);
            const uint32_t bf = P->dt_bit[ts] != kNoBit ? (v >> P->dt_bit[ts]) & 1u : P->base_bf16[ts];
            const uint32_t eb = bf ? 2u : 4u;
            uint32_t contig2, aligned2;
            tile_abstract(y, (uint32_t)S.d[1], (uint32_t)S.d[3], r2, c2, eb, strip, P->line_bytes, P->line_mask, qi[2 * ts], qi[2 * ts + 1],
                          contig2, aligned2);
            qc += contig2 * P->lim_stride[2 * ts] + aligned2 * P->lim_stride[2 * ts + 1];
          }
          off_c = ((combo * npass + pass) * Q + qc) * V + v;
        }
        const uint64_t sub = cost[(uint64_t)child * P->G + off_c];
        const bool fin = sub != kInf;
        const uint32_t a = te.trips;
        const uint64_t lo = (uint64_t)a * (uint32_t)sub;
        const uint64_t hi = (uint64_t)a * (uint32_t)(sub >> 32) + (lo >> 32);
        const uint64_t c = ((hi << 32) | (uint32_t)lo) + s;
        const bool over = fin & (((hi >> 30) != 0) | (c >= kLimit));
        e.ovf |= over ? 1u : 0u;
        consider(e, c, P->tile_base + (uint32_t)d * P->maxs + te.jt, fin & !over);
        e.n++;
      }
    }
    // bufferize (fused Spec): the Matmul into the intermediate at level `pass`, then the bias-add +
    // ReLU out of it; both read from the bounded tables of those two kinds
    if (P->kind == kKindF) {
      uint32_t qc = q;
      bool fits = true;
      const uint32_t la = P->lim_of_level[pass];
      if (la != kNoBit) {
        const uint32_t qa = la == 0 ? qi[0] : la == 1 ? qi[1] : la == 2 ? qi[2] : qi[3];
        const uint64_t bytes = S.numel[4] * 4u;
        const uint64_t have = qa ? 1ull << (qa - 1u) : 0ull;
        fits = bytes <= have;
        const uint64_t left = fits ? have - bytes : 0ull;
        const uint32_t qn = left ? 64u - (uint32_t)__clzll((long long)left) : 0u;
        qc = fits ? q - (qa - qn) * P->lim_stride[la] : q;
      }
      if (fits) {
        const uint32_t NL = P->NL;
        const uint32_t y0 = P->lay_bit[0] != kNoBit ? (v >> P->lay_bit[0]) & 1u : 0u;
        const uint32_t y1 = P->lay_bit[1] != kNoBit ? (v >> P->lay_bit[1]) & 1u : 0u;
        const uint32_t y3 = P->lay_bit[3] != kNoBit ? (v >> P->lay_bit[3]) & 1u : 0u;
        const uint32_t vm = (P->layM[0] != kNoBit ? y0 << P->layM[0] : 0u) + (P->layM[1] != kNoBit ? y1 << P->layM[1] : 0u);
        const uint32_t ve = P->layE[2] != kNoBit ? y3 << P->layE[2] : 0u;
        const uint32_t xm = (((lv[0] * NL + lv[1]) * NL + pass) * Q + qc) * P->VM + vm;
        const uint32_t xe = (((pass * NL + lv[2]) * NL + lv[3]) * Q + qc) * P->VE + ve;
        const uint64_t cm = P->costM[(uint64_t)((S.si[1] * P->nkM + S.si[2] + P->kM_first) * P->nsz[3] + S.si[3]) * P->GM + xm];
        const uint64_t ce = P->costE[(uint64_t)(S.si[1] * P->nszE_n + S.si[3]) * P->GE + xe];
        const uint32_t zc = pass == 0 ? P->zero[0] : pass == 1 ? P->zero[1] : pass == 2 ? P->zero[2] : P->zero[3];
        if (cm != kInf && ce != kInf) {
          const uint64_t z = mul_or_limit(zc, S.numel[4]);
          const uint64_t sum = z + cm;          // each term <= 2^62: no wrap
          if (z >= kLimit || sum >= kLimit || sum + ce >= kLimit) e.ovf = 1; else consider(e, sum + ce, P->buf_id);
        }
        e.n++;
      }
    }
    }   // admissible
    cost[group + off] = e.best;
    arg[group + off] = (uint16_t)e.arg;
  }
  // rewrites evaluated (and Specs that fit): one atomic each per workgroup
  uint32_t n_rw = e.n;
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) {
    n_rw += __shfl_down(n_rw, d, 64);
    if (MODE != 0) n_adm += __shfl_down(n_adm, d, 64);
  }
  if ((threadIdx.x & 63u) == 0) { wave_n[threadIdx.x >> 6] = n_rw; wave_adm[threadIdx.x >> 6] = n_adm; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t n = wave_n[0] + wave_n[1] + wave_n[2] + wave_n[3];
    if (n) atomicAdd(&ctr->n_rewrites[blockIdx.x % kCtrSlots], (unsigned long long)n);
    const uint32_t na = wave_adm[0] + wave_adm[1] + wave_adm[2] + wave_adm[3];
    if (MODE != 0 && na) atomicAdd(&ctr->n_admissible[blockIdx.x % kCtrSlots], (unsigned long long)na);
  }
  if (e.ovf) atomicOr(&ctr->overflow, e.ovf);
}

// One diagonal (or a part of it): n_blocks = segs.block0[segs.n].
void launch_fill_bounded(const DevParams* P, int mode, const uint32_t* all_level_shapes, const BoundSegs& segs, uint64_t* cost,
                         uint16_t* arg, Counters* ctr, hipStream_t stream) {
  if (!segs.n || !segs.block0[segs.n]) return;
  const dim3 grid(segs.block0[segs.n]);
  if (mode == 1) hipLaunchKernelGGL(fill_bounded_kernel<1>, grid, dim3(256), 0, stream, P, all_level_shapes, segs, cost, arg, ctr);
  else if (mode == 2) hipLaunchKernelGGL(fill_bounded_kernel<2>, grid, dim3(256), 0, stream, P, all_level_shapes, segs, cost, arg, ctr);
  else hipLaunchKernelGGL(fill_bounded_kernel<0>, grid, dim3(256), 0, stream, P, all_level_shapes, segs, cost, arg, ctr);
}

void launch_plan(const DevParams* P, uint32_t n_shapes, uint32_t npass, uint32_t G, const uint32_t* level_shapes,
                 const uint32_t* level_off, uint32_t n_levels, uint32_t* shape_class, uint32_t* list_whole,
                 uint32_t* list_slice, uint32_t* list_wide, uint32_t* list_cnt, uint32_t* fitmap, Counters* ctr,
                 void* prefill_cost, void* prefill_arg, hipStream_t stream) {
  const uint32_t cap = fill_wave_cap(G);
  hipLaunchKernelGGL(plan_kernel, dim3((n_shapes + 4 * kPlanShapes - 1) / (4 * kPlanShapes)), dim3(256), 0, stream, P,
                     n_shapes, cap, cap, kWaveCap < cap ? kWaveCap : cap, shape_class, fitmap, ctr, (uint4*)prefill_cost,
                     (uint4*)prefill_arg);
  hipLaunchKernelGGL(sort_work_kernel, dim3(n_levels), dim3(kSortThreads), 0, stream, level_shapes, level_off, n_levels, npass,
                     shape_class, list_whole, list_slice, list_wide, list_cnt);
}

// One dependency level: the items an LDS slice holds, and the wide ones (independent of each other:
// the caller may give them a stream of their own).  list_whole: the level's stretch of n_stretch
// entries, n_small small shapes at its front and n_bigwhole others at its back.
void launch_fill_level(const DevParams* P, uint32_t npass, uint32_t G, uint32_t max_task, const uint32_t* list_whole,
                       uint32_t n_stretch, uint32_t n_small, uint32_t n_bigwhole, const uint32_t* list_slice,
                       uint32_t n_slice, const uint32_t* list_wide, uint32_t n_wide, uint64_t* cost, uint16_t* arg,
                       Counters* ctr, hipStream_t stream, hipStream_t wide_stream) {
  const uint32_t cap = fill_wave_cap(G), n = n_bigwhole + n_slice + n_small;
  static const uint32_t wide_below = getenv("MRL_WIDE_BELOW") ? (uint32_t)atoi(getenv("MRL_WIDE_BELOW")) : kWideBelow;
  static const uint32_t big2_below = getenv("MRL_BIG2_BELOW") ? (uint32_t)atoi(getenv("MRL_BIG2_BELOW")) : 0u;
  if (n >= wide_below)
    hipLaunchKernelGGL(fill_kernel<64>, dim3(n), dim3(64), unit_lds_bytes(cap, npass), stream, P, list_whole, n_stretch,
                       n_bigwhole, list_slice, n_slice, cap, cost, arg, ctr);
  else if (n)
    hipLaunchKernelGGL(fill_kernel<256>, dim3(n), dim3(256), unit_lds_bytes(cap, npass), stream, P, list_whole, n_stretch,
                       n_bigwhole, list_slice, n_slice, cap, cost, arg, ctr);
  if (n_wide && n_wide < big2_below)
    hipLaunchKernelGGL(fill_big_kernel<2 * kBigBlock>, dim3(n_wide), dim3(2 * kBigBlock), unit_lds_bytes(max_task, npass), wide_stream, P,
                       list_wide, max_task, cost, arg, ctr);
  else if (n_wide)
    hipLaunchKernelGGL(fill_big_kernel<kBigBlock>, dim3(n_wide), dim3(kBigBlock), unit_lds_bytes(max_task, npass), wide_stream, P,
                       list_wide, max_task, cost, arg, ctr);
}

}  // namespace mrl
