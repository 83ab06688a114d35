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
//      (INF, NONE) by a plain streaming kernel, so this kernel writes the
//      admissible entries only;
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
// A shape with more tasks than the wave's LDS slice holds is appended to a
// list, one item per value of the passive level axis (the intermediate's level
// of a fused Spec: such slices are independent), and redone by a second launch
// with a whole workgroup per item and a slice sized for the largest possible
// item.  Nothing is reduced across lanes and no result depends on which wave
// handles a shape: the table is deterministic.
#include <hip/hip_runtime.h>
#include "compress.h"
#include "dev_params.h"

namespace mrl {

constexpr int kBatch = 8;              // sub-Spec costs fetched together before they are compared
constexpr uint32_t kSharedLds = 2048;  // Move cost table [convert][operand][src][dst][transposed], u64, per workgroup
constexpr uint32_t kSmallCap = 512;    // tasks a wave's LDS slice holds in the first launch
constexpr uint32_t kBigBlock = 512;    // threads per deferred item in the second launch
constexpr uint32_t kBigGrid = 1024;    // workgroups of the second launch (they loop over the deferred units)


struct Eval {
  uint64_t best;
  uint32_t arg;
  uint32_t n;
  uint32_t ovf;
};

__device__ __forceinline__ void consider(Eval& e, uint64_t cand, uint32_t id) {
  if (cand < e.best) { e.best = cand; e.arg = id; }
}

// a * sub + b with a < 2^32, sub < 2^62 (or INF, which is absorbing), b < 2^62.
// Two 32x32+64 multiply-adds give the 96-bit product; reaching 2^62 raises the overflow flag.
__device__ __forceinline__ uint64_t affine_mul(Eval& e, uint32_t a, uint64_t sub, uint64_t b) {
  if (sub == kInf) return kInf;
  const uint64_t lo = (uint64_t)a * (uint32_t)sub;
  const uint64_t hi = (uint64_t)a * (uint32_t)(sub >> 32) + (lo >> 32);   // bits 32.. of the product
  const uint64_t prod = (hi << 32) | (uint32_t)lo;
  if ((hi >> 30) != 0 || prod + b >= kLimit) { e.ovf = 1; return kInf; }
  return prod + b;
}

// sub + b, same conventions (b may be the sentinel kLimit for "coefficient * elements overflows").
__device__ __forceinline__ uint64_t affine_add(Eval& e, uint64_t sub, uint64_t b) {
  if (sub == kInf) return kInf;
  if (b >= kLimit || sub + b >= kLimit) { e.ovf = 1; return kInf; }
  return sub + b;
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
  else if (P->kind == kKindE) { S.numel[0] = m * n; S.numel[1] = n; S.numel[2] = m * n; S.numel[3] = 0; S.numel[4] = 0; }
  else { S.numel[0] = m * k; S.numel[1] = k * n; S.numel[2] = n; S.numel[3] = m * n; S.numel[4] = m * n; }
}

__device__ __forceinline__ uint32_t level_of(const DevParams* __restrict__ P, uint32_t pack, int i) {
  return (pack >> P->pack_shift[i]) & 3u;
}

__device__ __forceinline__ uint32_t combo_of_pack(const DevParams* __restrict__ P, uint32_t pack) {
  if (P->NL == 4) return pack;
  uint32_t c = 0;
#pragma unroll
  for (int i = 0; i < 4; i++) if ((uint32_t)i < P->nops) c += level_of(P, pack, i) * P->lvpow[i];
  return c;
}

__device__ __forceinline__ uint32_t pack_of_combo(const DevParams* __restrict__ P, uint32_t combo) {
  if (P->NL == 4) return combo;
  uint32_t p = 0;
  if (P->level_bits != 0xFF) {
#pragma unroll
    for (int i = 0; i < 4; i++)
      if ((uint32_t)i < P->nops) p |= ((combo >> (P->level_bits * (P->nops - 1 - i))) & (P->NL - 1)) << P->pack_shift[i];
  } else {
#pragma unroll
    for (int i = 0; i < 4; i++) if ((uint32_t)i < P->nops) p |= ((combo / P->lvpow[i]) % P->NL) << P->pack_shift[i];
  }
  return p;
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
      const uint32_t bf = P->dt_bit[i] != 0xFF ? (dt >> P->dt_bit[i]) & 1u : P->base_bf16[i];
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
__device__ __forceinline__ uint32_t admissible_mask(const DevParams* __restrict__ P, const uint32_t* fit,
                                                    uint32_t info, uint32_t pass) {
  const uint32_t ndtpat = 1u << P->ndt;
  const bool fused = P->kind == kKindF;
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
    default: return 0;
  }
}

// LDS of one unit (a shape, or one passive-level slice of it).  "xpack" = pass<<8 | pack.
struct UnitLds {
  uint64_t* t_cost;   // [cap] per task: best tile/bufferize candidate, then the final cost
  uint32_t* t_spec;   // [cap] xpack | variant<<10 | id<<16
  uint32_t* c_info;   // [npass*256] by xpack: admissible variants (low 16 bits) | first task << 16
  uint32_t* r_off;    // [nranks+1] first task of the rank
  uint32_t* wave_tot; // [16] scan scratch
  uint32_t* fit;      // [16] see build_fit
};

__host__ __device__ inline uint32_t unit_lds_bytes(uint32_t cap, uint32_t npass) {
  return (cap * 12u + npass * 1024u + (kMaxRanks + 2) * 4u + 32u * 4u + 15u) & ~15u;
}

__device__ __forceinline__ UnitLds carve(unsigned char* w, uint32_t cap, uint32_t npass) {
  UnitLds L;
  L.t_cost = reinterpret_cast<uint64_t*>(w);
  L.t_spec = reinterpret_cast<uint32_t*>(L.t_cost + cap);
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

// Move cost per (convert, operand, src, dst, transposed) for this shape: coefficient * elements.
template <int T>
__device__ __forceinline__ void build_move_costs(const DevParams* __restrict__ P, const Shape& S, uint64_t* bterm) {
  for (uint32_t e = T == 64 ? (threadIdx.x & 63u) : threadIdx.x; e < 256; e += T) {
    const uint32_t cv = e >> 7, i = (e >> 5) & 3u;
    const uint32_t c = (&P->mcoef[0][0][0][0])[e & 127u];
    const uint64_t n = i == 0 ? S.numel[0] : i == 1 ? S.numel[1] : i == 2 ? S.numel[2] : S.numel[3];
    bterm[e] = c ? mul_or_limit((uint64_t)c + (cv ? P->convert : 0u), n) : 0;   // 0 = the Move does not exist
  }
}

// Step 3 for task q: tile and bufferize candidates.
__device__ __forceinline__ void task_tiles(const DevParams* __restrict__ P, const UnitLds& L, const Shape& S,
                                           uint32_t shape, uint32_t q, const uint64_t* __restrict__ cost, Eval& tot) {
  const uint32_t V = P->V, npass = P->npass, NL = P->NL;
  const uint32_t sp = L.t_spec[q];
  const uint32_t pack = sp & 0xFFu, pass = (sp >> 8) & 3u, v = (sp >> 10) & 31u;
  const uint32_t off = (combo_of_pack(P, pack) * npass + pass) * V + v;
  Eval e;
  e.best = kInf; e.arg = kNone; e.n = 0; e.ovf = 0;
#pragma unroll
  for (int d = 0; d < 4; d++) {
    if (!P->tile_dim_ok[d]) continue;
    const uint32_t j = S.si[d];
    const uint32_t q_end = P->tile_off[d][j + 1];
    e.n += q_end - P->tile_off[d][j];
    for (uint32_t q2 = P->tile_off[d][j]; q2 < q_end; q2 += kBatch) {
      uint64_t sub[kBatch];
      uint32_t jt[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; u++) {
        const uint32_t qq = q2 + u < q_end ? q2 + u : q_end - 1;
        jt[u] = P->tile_jt[qq];
        sub[u] = cost[(uint64_t)(shape - (j - jt[u]) * P->shape_stride[d]) * P->G + off];
      }
#pragma unroll
      for (int u = 0; u < kBatch; u++)
        if (q2 + u < q_end)
          consider(e, affine_mul(e, P->tile_trips[q2 + u], sub[u], P->s), P->tile_base + d * P->maxs + jt[u]);
    }
  }
  // bufferize (FUSED): Matmul into the intermediate, then bias-add+ReLU out of it
  if (P->kind == kKindF) {
    const uint32_t l0 = level_of(P, pack, 0), l1 = level_of(P, pack, 1), l2 = level_of(P, pack, 2), l3 = level_of(P, pack, 3);
    const uint32_t y0 = P->lay_bit[0] != 0xFF ? (v >> P->lay_bit[0]) & 1u : 0u;
    const uint32_t y1 = P->lay_bit[1] != 0xFF ? (v >> P->lay_bit[1]) & 1u : 0u;
    const uint32_t y3 = P->lay_bit[3] != 0xFF ? (v >> P->lay_bit[3]) & 1u : 0u;
    const uint32_t xm = ((l0 * NL + l1) * NL + pass) * P->VM +
                        (P->layM[0] != 0xFF ? y0 << P->layM[0] : 0u) + (P->layM[1] != 0xFF ? y1 << P->layM[1] : 0u);
    const uint32_t xe = ((pass * NL + l2) * NL + l3) * P->VE + (P->layE[2] != 0xFF ? y3 << P->layE[2] : 0u);
    const uint64_t cm = P->costM[(uint64_t)shape * P->GM + xm];
    const uint64_t ce = P->costE[(uint64_t)(S.si[1] * P->nszE_n + S.si[3]) * P->GE + xe];
    const uint32_t zc = pass == 0 ? P->zero[0] : pass == 1 ? P->zero[1] : pass == 2 ? P->zero[2] : P->zero[3];
    uint64_t cand = kInf;
    if (cm != kInf && ce != kInf) {
      const uint64_t z = mul_or_limit(zc, S.numel[4]);
      const uint64_t sum = z + cm;          // each term <= 2^62: no wrap
      if (z >= kLimit || sum >= kLimit || sum + ce >= kLimit) e.ovf = 1; else cand = sum + ce;
    }
    consider(e, cand, P->buf_id);
    e.n += 1;
  }
  L.t_cost[q] = e.best;
  L.t_spec[q] = sp | e.arg << 16;
  tot.n += e.n;
  tot.ovf |= e.ovf;
}

// Step 4 for task q (all sub-Specs of lower rank are final in LDS).
__device__ __forceinline__ void task_rank(const DevParams* __restrict__ P, const UnitLds& L, const uint64_t* bterm,
                                          const Shape& S, uint64_t group, uint32_t q, uint32_t mk_shape,
                                          uint64_t* __restrict__ cost, uint16_t* __restrict__ arg, Eval& tot) {
  const uint32_t V = P->V, n_slots = P->n_slots;
  const bool has_dt = P->ndt != 0;
  const uint32_t sp = L.t_spec[q];
  const uint32_t xpack = sp & 0x3FFu, v = (sp >> 10) & 31u;
  Eval e;
  e.best = kInf; e.arg = kNone; e.n = 0; e.ovf = 0;
  uint32_t hi_or = 0;       // OR of the high words of all finite candidates: bit 30 set <=> one reached 2^62

  // A. select(microkernel)
  if (mk_shape) {
    for (uint32_t mm = P->mk_entry[(xpack & 0xFFu) * V + v] & mk_shape; mm; mm &= mm - 1) {
      const uint32_t j = (uint32_t)__ffs(mm) - 1u;
      const uint64_t k = mul_or_limit(P->mk_cost[j], mk_shape_reps(P, S, j));
      if (k >= kLimit) e.ovf = 1; else consider(e, k, j);
      e.n++;
    }
  }

  // B. Move an operand to a strictly lower level: kBatch LDS lookups in flight
  for (uint32_t s0 = 0; s0 < n_slots; s0 += kBatch) {
    uint64_t cand[kBatch];
    uint32_t id[kBatch];
    bool ok[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; u++) {
      const uint32_t sl = P->slots[s0 + u < n_slots ? s0 + u : n_slots - 1];
      const uint32_t dst = (sl >> 2) & 3u, cv = (sl >> 5) & 1u, sh = (sl >> 6) & 7u, dtb = (sl >> 12) & 7u;
      const uint32_t b_idx = cv * 128u + (sl & 3u) * 32u + dst * 2u + ((sl >> 4) & 1u);   // + src * 8
      const uint32_t v_xor = ((sl >> 4) & 1u) << ((sl >> 9) & 7u), v_clr = cv << dtb;
      const uint32_t src = (xpack >> sh) & 3u;
      const uint64_t b = bterm[b_idx + src * 8u];
      bool valid = s0 + u < n_slots && dst < src && b != 0;
      if (has_dt) valid = valid && (!cv || ((v >> dtb) & 1u));
      const uint32_t xp2 = valid ? xpack - ((src - dst) << sh) : xpack;
      const uint32_t v2 = (v ^ v_xor) & ~v_clr;
      const uint32_t ci = L.c_info[xp2];
      const bool has = valid && ((ci >> v2) & 1u);
      const uint32_t idx = (ci >> 16) + (has_dt ? __popc(ci & 0xFFFFu & ((1u << v2) - 1u)) : v2);
      const uint64_t t = L.t_cost[has ? idx : q];
      const bool fin = has && t != kInf;
      const uint64_t c = t + b;            // t < 2^62 when finite, b <= 2^62: no wrap
      cand[u] = fin ? c : kInf;
      hi_or |= fin ? (uint32_t)(c >> 32) : 0u;
      id[u] = sl >> 16;
      ok[u] = valid;
    }
#pragma unroll
    for (int u = 0; u < kBatch; u++)
      if (ok[u]) { consider(e, cand[u], id[u]); e.n++; }
  }
  if (hi_or >> 30) {          // some finite candidate reached 2^62: the whole solve reports overflow
    e.ovf = 1;
  }

  // C, D. tiles and bufferize, evaluated in step 3
  const uint64_t tb = L.t_cost[q];
  if (tb < e.best) { e.best = tb; e.arg = sp >> 16; }

  const uint32_t off = (combo_of_pack(P, xpack & 0xFFu) * P->npass + (xpack >> 8)) * V + v;
  L.t_cost[q] = e.best;
  cost[group + off] = e.best;
  arg[group + off] = (uint16_t)e.arg;
  tot.n += e.n;
  tot.ovf |= e.ovf;
}

// One unit = passes [pass0, pass0 + np) of one shape, handled by T threads
// (T = 64: the wave of the first launch, all passes; T = kBigBlock: the second launch, one pass).
template <int T, bool BIG>
__device__ __forceinline__ void solve_unit(const DevParams* __restrict__ P, uint64_t* bterm, const UnitLds& L,
                                           uint32_t cap, const Shape& S, uint32_t shape, uint32_t pass0, uint32_t np,
                                           uint32_t* __restrict__ big_list, uint32_t* __restrict__ big_count,
                                           uint64_t* __restrict__ cost, uint16_t* __restrict__ arg,
                                           Eval& tot, uint32_t& n_adm) {
  const uint32_t tid = T == 64 ? (threadIdx.x & 63u) : threadIdx.x;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t npass = P->npass;
  const uint64_t group = (uint64_t)shape * P->G;

  // ---- 1. admissibility, compaction in rank order (rank-major level assignments, then pass) ----
  if (threadIdx.x < 64) build_fit(P, S, L.fit);
  unit_sync<T>();
  uint32_t n_task = 0;
  for (uint32_t p0 = 0; p0 < P->ncombo; p0 += T) {
    const uint32_t pc = p0 + tid;
    uint32_t mask[4] = {0, 0, 0, 0}, info = 0, cnt = 0;
    if (pc < P->ncombo) {
      info = P->pos_info[pc];
#pragma unroll
      for (int ps = 0; ps < 4; ps++)
        if ((uint32_t)ps < np) { mask[ps] = admissible_mask(P, L.fit, info, pass0 + ps); cnt += __popc(mask[ps]); }
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
    if (pc < P->ncombo) {
#pragma unroll
      for (int ps = 0; ps < 4; ps++)
        if ((uint32_t)ps < np) {
          const uint32_t xpack = (pass0 + ps) << 8 | (info & 0xFFu);
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
  if (n_task == 0) return;          // nothing of this shape fits anywhere: the table already says so
  unit_sync<T>();
  if (tid <= P->nranks)
    L.r_off[tid] = tid == P->nranks ? n_task : L.c_info[pass0 << 8 | P->pack_by_rank[P->rank_off[tid]]] >> 16;
  build_move_costs<T>(P, S, bterm);
  unit_sync<T>();

  if (!BIG) {
    n_adm += tid == 0 ? n_task : 0;
    if (n_task > cap) {          // too many tasks for the wave's LDS slice: leave the shape to the second launch
      if (tid < npass) big_list[atomicAdd(big_count, 1u)] = shape * npass + tid;
      return;
    }
  }

  // ---- 3. tile and bufferize candidates of every task ----
  for (uint32_t q = tid; q < n_task; q += T) task_tiles(P, L, S, shape, q, cost, tot);
  unit_sync<T>();

  // microkernels whose shape predicate holds for this shape (uniform)
  uint32_t mk_shape = 0;
  for (uint32_t j = 0; j < P->nmk; j++) mk_shape |= (mk_shape_reps(P, S, j) ? 1u : 0u) << j;

  // ---- 4. rank by rank ----
  for (uint32_t r = 0; r < P->nranks; r++) {
    const uint32_t t0 = L.r_off[r], t1 = L.r_off[r + 1];
    if (t0 == t1) continue;
    for (uint32_t q = t0 + tid; q < t1; q += T) task_rank(P, L, bterm, S, group, q, mk_shape, cost, arg, tot);
    unit_sync<T>();
  }
}

__device__ __forceinline__ void flush_counters(Counters* __restrict__ ctr, const Eval& tot, uint32_t n_adm) {
  uint32_t n_rw = tot.n;
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) n_rw += __shfl_down(n_rw, d, 64);
  if ((threadIdx.x & 63u) == 0) {
    if (n_rw) atomicAdd(&ctr->n_rewrites, (unsigned long long)n_rw);
    if (n_adm) atomicAdd(&ctr->n_admissible, (unsigned long long)n_adm);
  }
  if (tot.ovf) atomicOr(&ctr->overflow, 1u);
}

// First launch of a level: one wave per shape.
__global__ __launch_bounds__(64) void fill_kernel(const DevParams* __restrict__ P,
                                                  const uint32_t* __restrict__ level_shapes,
                                                  uint32_t* __restrict__ big_list, uint32_t* __restrict__ big_count,
                                                  uint32_t cap, uint64_t* __restrict__ cost,
                                                  uint16_t* __restrict__ arg, Counters* __restrict__ ctr) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint64_t* bterm = reinterpret_cast<uint64_t*>(smem);
  const uint32_t shape = level_shapes[blockIdx.x];
  Shape S;
  load_shape(P, shape, S);
  const UnitLds L = carve(smem + kSharedLds, cap, P->npass);
  Eval tot;
  tot.n = 0; tot.ovf = 0;
  uint32_t n_adm = 0;
  solve_unit<64, false>(P, bterm, L, cap, S, shape, 0, P->npass, big_list, big_count, cost, arg, tot, n_adm);
  flush_counters(ctr, tot, n_adm);
}

// Second launch of a level: the deferred items, one workgroup of kBigBlock threads each.
__global__ __launch_bounds__(kBigBlock) void fill_big_kernel(const DevParams* __restrict__ P,
                                                             uint32_t* __restrict__ big_list,
                                                             uint32_t* __restrict__ big_count, uint32_t cap,
                                                             uint64_t* __restrict__ cost, uint16_t* __restrict__ arg,
                                                             Counters* __restrict__ ctr) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint64_t* bterm = reinterpret_cast<uint64_t*>(smem);
  const UnitLds L = carve(smem + kSharedLds, cap, P->npass);
  Eval tot;
  tot.n = 0; tot.ovf = 0;
  uint32_t n_adm = 0;
  const uint32_t n_units = *big_count;
  for (uint32_t u = blockIdx.x; u < n_units; u += gridDim.x) {
    const uint32_t unit = big_list[u];
    const uint32_t shape = unit / P->npass, pass = unit % P->npass;
    Shape S;
    load_shape(P, shape, S);
    __syncthreads();            // the previous item's LDS is dead
    solve_unit<kBigBlock, true>(P, bterm, L, cap, S, shape, pass, 1, big_list, big_count, cost, arg, tot, n_adm);
  }
  flush_counters(ctr, tot, n_adm);
}

// (INF, NONE) are all-ones bytes: stream 16 bytes per lane and store over both tables.
__global__ __launch_bounds__(256) void fill_ones_kernel(uint4* __restrict__ p, size_t n16) {
  const uint4 ones = make_uint4(~0u, ~0u, ~0u, ~0u);
  for (size_t i = (size_t)blockIdx.x * 256u + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256u) p[i] = ones;
}

void launch_fill_ones(void* p, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;       // tables are 256-byte aligned and hold a multiple of 16 bytes... or a tail
  if (n16) {
    const size_t blocks = (n16 + 255) / 256;
    hipLaunchKernelGGL(fill_ones_kernel, dim3((uint32_t)(blocks < 16384 ? blocks : 16384)), dim3(256), 0, stream,
                       (uint4*)p, n16);
  }
  if (bytes % 16) (void)hipMemsetAsync((char*)p + n16 * 16, 0xFF, bytes % 16, stream);
}

// One dependency level: every shape by the first kernel, then the items it deferred.
void launch_fill_level(const DevParams* P, uint32_t npass, uint32_t G, uint32_t max_task, const uint32_t* level_shapes,
                       uint32_t n_shapes, uint32_t* big_list, uint32_t* big_count, uint64_t* cost, uint16_t* arg,
                       Counters* ctr, hipStream_t stream) {
  if (n_shapes == 0) return;
  const uint32_t small_cap = G < kSmallCap ? G : kSmallCap;
  hipLaunchKernelGGL(fill_kernel, dim3(n_shapes), dim3(64), kSharedLds + unit_lds_bytes(small_cap, npass), stream, P,
                     level_shapes, big_list, big_count, small_cap, cost, arg, ctr);
  if (G > small_cap) {
    const uint32_t units = n_shapes * npass;
    hipLaunchKernelGGL(fill_big_kernel, dim3(units < kBigGrid ? units : kBigGrid), dim3(kBigBlock),
                       kSharedLds + unit_lds_bytes(max_task, npass), stream, P, big_list, big_count, max_task, cost, arg,
                       ctr);
  }
}

}  // namespace mrl
