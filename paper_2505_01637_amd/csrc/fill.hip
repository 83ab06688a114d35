// Rewrite evaluation + argmin for one dependency level of the Spec lattice.
//
// Paper, Section 4: a Spec's entry is the lowest-cost applicable rewrite, the
// rewrite's cost being the affine function of Section 3 of its sub-Specs'
// costs.  Here the table is filled bottom-up: all shapes of one dependency
// level in one launch, every sub-Spec of another shape already final.
//
// Mapping (gfx950, wave64).  A workgroup owns one *unit*: one shape (b,m,k,n)
// and one value of the passive level axis; a unit is closed under Moves.
//   1. one thread per operand-level combo decides which entries fit their
//      levels and the admissible ones are compacted, ordered by rank (sum of
//      the operand levels), into a task list in LDS;
//   2. entries that do not fit are streamed out as (INF, NONE);
//   3. one thread per task evaluates the tile and bufferize rewrites, whose
//      sub-Specs belong to other shapes or tables and are final: a tile
//      sub-Spec sits at the same offset of a smaller shape's group, so
//      consecutive lanes read consecutive addresses, several loads in flight
//      per lane.  The best of them is parked in LDS;
//   4. rank by rank, one thread per task evaluates the microkernels and the
//      Moves (sub-Specs in the same unit at a lower rank: read from LDS), in
//      id order, keeping the first strict minimum (= lowest id among ties),
//      then takes the parked candidate if strictly lower (its ids are higher).
//      Results go to LDS (for later ranks) and to the table.
// Nothing is reduced across lanes, so the result cannot depend on timing.
#include <hip/hip_runtime.h>
#include "dev_params.h"

namespace mrl {

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

// Exclusive prefix sum of one value per thread over the workgroup (T = 64 or 256).
template <int T>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total) {
  uint32_t incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t o = __shfl_up(incl, d, 64);
    if ((int)lane_id() >= d) incl += o;
  }
  if (T == 64) {
    *total = __shfl(incl, 63, 64);
    return incl - v;
  }
  uint32_t w = threadIdx.x >> 6;
  if (lane_id() == 63) wave_tot[w] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < T / 64; i++) {
    uint32_t t = wave_tot[i];
    if ((uint32_t)i < w) base += t;
    tot += t;
  }
  *total = tot;
  return base + incl - v;
}

struct Eval {
  uint64_t best;
  uint32_t arg;
  uint32_t n;
  uint32_t ovf;
};

__device__ __forceinline__ void consider(Eval& e, uint64_t cand, uint32_t id) {
  e.n++;
  if (cand < e.best) { e.best = cand; e.arg = id; }
}

// a * sub + b, INF absorbing; anything reaching 2^62 raises the overflow flag.
__device__ __forceinline__ uint64_t affine(Eval& e, uint64_t a, uint64_t sub, uint64_t b) {
  if (sub == kInf) return kInf;
  uint64_t lo = a * sub;
  if (__umul64hi(a, sub) != 0 || lo >= kLimit || b >= kLimit || lo + b >= kLimit) { e.ovf = 1; return kInf; }
  return lo + b;
}

__device__ __forceinline__ uint64_t mul_checked(Eval& e, uint64_t a, uint64_t b) {
  uint64_t lo = a * b;
  if (__umul64hi(a, b) != 0 || lo >= kLimit) { e.ovf = 1; return kLimit; }
  return lo;
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

__device__ __forceinline__ void decode_levels(const DevParams* __restrict__ P, uint32_t combo, uint32_t lv[4]) {
#pragma unroll
  for (int i = 0; i < 4; i++) lv[i] = (uint32_t)i < P->nops ? (combo / P->lvpow[i]) % P->NL : 0u;
}

// Bit v of the result: variant v of this combo fits every level's capacity.
__device__ __forceinline__ uint32_t admissible_mask(const DevParams* __restrict__ P, const Shape& S,
                                                    const uint32_t lv[4], uint32_t pass) {
  uint32_t ndtpat = 1u << P->ndt;
  uint32_t bits = 0;
  for (uint32_t dt = 0; dt < ndtpat; dt++) {
    uint64_t used[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 4; i++) {
      if ((uint32_t)i >= P->nops) break;
      uint32_t bf = P->dt_bit[i] != 0xFF ? (dt >> P->dt_bit[i]) & 1u : P->base_bf16[i];
      uint64_t bytes = S.numel[i] * (bf ? 2u : 4u);
#pragma unroll
      for (int l = 0; l < 4; l++) used[l] += lv[i] == (uint32_t)l ? bytes : 0;
    }
    if (P->kind == kKindF) {
#pragma unroll
      for (int l = 0; l < 4; l++) used[l] += pass == (uint32_t)l ? S.numel[4] * 4u : 0;
    }
    bool ok = true;
#pragma unroll
    for (int l = 0; l < 4; l++) ok = ok && ((uint32_t)l >= P->NL || used[l] <= P->cap[l]);
    bits |= (ok ? 1u : 0u) << dt;
  }
  uint32_t mask = 0;
  for (uint32_t lay = 0; lay < (1u << P->nlay); lay++) mask |= bits << (lay * ndtpat);
  return mask;
}

// Number of repetitions of microkernel j on this Spec, 0 if its predicate fails
// (Section 2, Microkernel Selection; Figure 1 for BroadcastVecMultAdd).
__device__ __forceinline__ uint64_t mk_reps(const DevParams* __restrict__ P, const Shape& S, uint32_t j,
                                            const uint32_t lv[4], const uint32_t ly[4], const uint32_t bf[4]) {
  uint64_t b = S.d[0], m = S.d[1], k = S.d[2], n = S.d[3];
  uint32_t lanes = P->mk_lanes[j];
  switch (P->mk_kind[j]) {
    case 0:
      if (P->kind != kKindM || b != 1 || m != 1 || k != 1 || n != 1) return 0;
      if (lv[0] | lv[1] | lv[2] | bf[0] | bf[1] | bf[2]) return 0;
      return 1;
    case 1:
      if (P->kind != kKindM || b != 1 || m != 1 || k != 1 || n % lanes) return 0;
      if (lv[0] != 0 || lv[1] != 1 || lv[2] != 1 || (bf[0] | bf[1] | bf[2]) || ly[1] || ly[2]) return 0;
      return n / lanes;
    case 2:
      if (P->kind != kKindM || b != 1 || m != 1 || n != 1 || k % lanes) return 0;
      if (lv[0] != 1 || lv[1] != 1 || lv[2] != 0 || !bf[0] || !bf[1] || bf[2]) return 0;
      if (P->lay_bit[1] != 0xFF && ly[1] != 1) return 0;
      return k / lanes;
    case 3:
      if (P->kind != kKindE || m != 1 || n != 1 || (lv[0] | lv[1] | lv[2])) return 0;
      return 1;
    case 4:
      if (P->kind != kKindE || m != 1 || n % lanes) return 0;
      if (lv[0] != 1 || lv[1] != 1 || lv[2] != 1 || ly[0] || ly[2]) return 0;
      return n / lanes;
    default: return 0;
  }
}

// Store `bytes` (2, 4, 8 or 16) bytes of all-ones at p: INF costs and NONE ids are all-ones.
__device__ __forceinline__ void store_ones(void* p, uint32_t bytes) {
  if (bytes == 16) *reinterpret_cast<uint4*>(p) = make_uint4(~0u, ~0u, ~0u, ~0u);
  else if (bytes == 8) *reinterpret_cast<uint2*>(p) = make_uint2(~0u, ~0u);
  else if (bytes == 4) *reinterpret_cast<uint32_t*>(p) = ~0u;
  else *reinterpret_cast<uint16_t*>(p) = (uint16_t)0xFFFFu;
}

constexpr int kTileBatch = 8;   // sub-Spec costs fetched together before they are compared

template <int T>
__global__ __launch_bounds__(T) void fill_level_kernel(const DevParams* __restrict__ P,
                                                        const uint32_t* __restrict__ level_shapes,
                                                        uint32_t n_units,
                                                        uint64_t* __restrict__ cost,
                                                        uint16_t* __restrict__ arg,
                                                        Counters* __restrict__ ctr) {
  extern __shared__ __align__(16) unsigned char smem[];
  const uint32_t ncombo = P->ncombo, V = P->V, npass = P->npass;
  const uint32_t max_task = ncombo * V;
  uint64_t* t_cost = reinterpret_cast<uint64_t*>(smem);                  // [max_task] per task: best tile/bufferize
                                                                          //   candidate, then the final cost
  uint32_t* t_spec = reinterpret_cast<uint32_t*>(t_cost + max_task);     // [max_task] combo | variant<<8 | id<<16
  uint32_t* c_mask = t_spec + max_task;                                   // [ncombo] admissible variants
  uint32_t* c_base = c_mask + ncombo;                                     // [ncombo] first task of the combo
  uint32_t* r_off = c_base + ncombo;                                      // [nranks+1] first task of the rank
  uint32_t* wave_tot = r_off + kMaxRanks + 2;                             // [4]

  const uint32_t unit = blockIdx.x;
  if (unit >= n_units) return;
  const uint32_t shape = level_shapes[unit / npass];
  const uint32_t pass = unit % npass;
  const uint32_t tid = threadIdx.x;

  Shape S;
  load_shape(P, shape, S);
  const uint64_t group = (uint64_t)shape * P->G;

  // ---- 1. admissibility, compaction in rank order ----
  uint32_t my_mask = 0, my_combo = 0;
  if (tid < ncombo) {
    my_combo = P->combo_by_rank[tid];
    uint32_t lv[4];
    decode_levels(P, my_combo, lv);
    my_mask = admissible_mask(P, S, lv, pass);
    c_mask[my_combo] = my_mask;
  }
  uint32_t n_task;
  uint32_t my_base = block_exclusive_scan<T>(__popc(my_mask), wave_tot, &n_task);
  if (tid < ncombo) {
    c_base[my_combo] = my_base;
    uint32_t q = my_base;
    for (uint32_t m = my_mask; m; m &= m - 1) t_spec[q++] = my_combo | ((uint32_t)__ffs(m) - 1u) << 8;
    for (uint32_t r = 0; r < P->nranks; r++)
      if (tid == P->rank_off[r]) r_off[r] = my_base;
  }
  if (tid == 0) r_off[P->nranks] = n_task;
  __syncthreads();

  // ---- 2. entries that do not fit: (INF, NONE), written in chunks of up to 16 bytes ----
  {
    const uint32_t cch = V < 2 ? V : 2, cper = V / cch;        // cost: entries per chunk, chunks per combo
    for (uint32_t c = tid; c < ncombo * cper; c += T) {
      const uint32_t combo = c / cper, v0 = (c - combo * cper) * cch;
      const uint32_t bits = (c_mask[combo] >> v0) & ((1u << cch) - 1u);
      uint64_t* p = cost + group + (uint64_t)(combo * npass + pass) * V + v0;
      if (bits == 0) store_ones(p, 8 * cch);
      else for (uint32_t u = 0; u < cch; u++) if (!((bits >> u) & 1u)) p[u] = kInf;
    }
    const uint32_t ach = V < 8 ? V : 8, aper = V / ach;        // argmin: likewise
    for (uint32_t c = tid; c < ncombo * aper; c += T) {
      const uint32_t combo = c / aper, v0 = (c - combo * aper) * ach;
      const uint32_t bits = (c_mask[combo] >> v0) & ((1u << ach) - 1u);
      uint16_t* p = arg + group + (uint64_t)(combo * npass + pass) * V + v0;
      if (bits == 0) store_ones(p, 2 * ach);
      else for (uint32_t u = 0; u < ach; u++) if (!((bits >> u) & 1u)) p[u] = (uint16_t)kNone;
    }
  }

  Eval tot;
  tot.n = 0; tot.ovf = 0;
  const uint32_t NL = P->NL;

  // ---- 3. tile and bufferize candidates of every task (sub-Specs of other shapes / tables:
  //         final already, no ordering needed).  kTileBatch loads are in flight per thread. ----
  for (uint32_t q = tid; q < n_task; q += T) {
    const uint32_t sp = t_spec[q];
    const uint32_t combo = sp & 0xFFu, v = (sp >> 8) & 0xFFu;
    const uint32_t off = (combo * npass + pass) * V + v;
    Eval e;
    e.best = kInf; e.arg = kNone; e.n = 0; e.ovf = 0;
#pragma unroll
    for (int d = 0; d < 4; d++) {
      if (!P->tile_dim_ok[d]) continue;
      const uint32_t j = S.si[d];
      const uint32_t q_end = P->tile_off[d][j + 1];
      for (uint32_t q2 = P->tile_off[d][j]; q2 < q_end; q2 += kTileBatch) {
        uint64_t sub[kTileBatch];
        uint32_t jt[kTileBatch];
#pragma unroll
        for (int u = 0; u < kTileBatch; u++) {
          const uint32_t qq = q2 + u < q_end ? q2 + u : q_end - 1;
          jt[u] = P->tile_jt[qq];
          sub[u] = cost[(uint64_t)(shape - (j - jt[u]) * P->shape_stride[d]) * P->G + off];
        }
#pragma unroll
        for (int u = 0; u < kTileBatch; u++)
          if (q2 + u < q_end)
            consider(e, affine(e, P->tile_trips[q2 + u], sub[u], P->s), P->tile_base + d * P->maxs + jt[u]);
      }
    }
    // bufferize (FUSED): Matmul into the intermediate, then bias-add+ReLU out of it
    if (P->kind == kKindF) {
      uint32_t lv[4];
      decode_levels(P, combo, lv);
      const uint32_t y0 = P->lay_bit[0] != 0xFF ? (v >> P->lay_bit[0]) & 1u : 0u;
      const uint32_t y1 = P->lay_bit[1] != 0xFF ? (v >> P->lay_bit[1]) & 1u : 0u;
      const uint32_t y3 = P->lay_bit[3] != 0xFF ? (v >> P->lay_bit[3]) & 1u : 0u;
      const uint32_t xm = ((lv[0] * NL + lv[1]) * NL + pass) * P->VM +
                          (P->layM[0] != 0xFF ? y0 << P->layM[0] : 0u) + (P->layM[1] != 0xFF ? y1 << P->layM[1] : 0u);
      const uint32_t xe = ((pass * NL + lv[2]) * NL + lv[3]) * P->VE + (P->layE[2] != 0xFF ? y3 << P->layE[2] : 0u);
      const uint64_t cm = P->costM[(uint64_t)shape * P->GM + xm];
      const uint64_t ce = P->costE[(uint64_t)(S.si[1] * P->nszE_n + S.si[3]) * P->GE + xe];
      uint64_t cand = kInf;
      if (cm != kInf && ce != kInf) {
        const uint64_t z = mul_checked(e, P->zero[pass], S.numel[4]);
        const uint64_t sum = z + cm;          // each term < 2^62: no wrap
        if (sum >= kLimit || sum + ce >= kLimit) e.ovf = 1; else cand = sum + ce;
      }
      consider(e, cand, P->buf_id);
    }
    t_cost[q] = e.best;
    t_spec[q] = sp | e.arg << 16;
    tot.n += e.n;
    tot.ovf |= e.ovf;
  }
  __syncthreads();

  // ---- 4. rank by rank: microkernels, Moves (sub-Specs of lower rank, in LDS), then the
  //         stored tile/bufferize candidate, whose ids are higher: it wins only if strictly lower ----
  for (uint32_t r = 0; r < P->nranks; r++) {
    const uint32_t t0 = r_off[r], t1 = r_off[r + 1];
    if (t0 == t1) continue;
    for (uint32_t q = t0 + tid; q < t1; q += T) {
      const uint32_t sp = t_spec[q];
      const uint32_t combo = sp & 0xFFu, v = (sp >> 8) & 0xFFu;
      uint32_t lv[4], ly[4], bf[4];
      decode_levels(P, combo, lv);
#pragma unroll
      for (int i = 0; i < 4; i++) {
        ly[i] = P->lay_bit[i] != 0xFF ? (v >> P->lay_bit[i]) & 1u : 0u;
        bf[i] = P->dt_bit[i] != 0xFF ? (v >> P->dt_bit[i]) & 1u : P->base_bf16[i];
      }
      Eval e;
      e.best = kInf; e.arg = kNone; e.n = 0; e.ovf = 0;

      // A. select(microkernel)
      for (uint32_t j = 0; j < P->nmk; j++) {
        uint64_t reps = mk_reps(P, S, j, lv, ly, bf);
        if (reps) consider(e, affine(e, 0, 0, mul_checked(e, P->mk_cost[j], reps)), j);
      }

      // B. Move operand i to a strictly lower level
#pragma unroll
      for (int i = 0; i < 4; i++) {
        if ((uint32_t)i >= P->nops) break;
        const uint32_t src = lv[i], acc = P->access[i];
        for (uint32_t dst = 0; dst < src; dst++)
          for (uint32_t x = 0; x < 2; x++)
            for (uint32_t cv = 0; cv < 2; cv++) {
              if (x && P->lay_bit[i] == 0xFF) continue;
              if (cv && !(P->dt_bit[i] != 0xFF && bf[i] && acc == kRead)) continue;
              uint64_t coef = 0;
              if (acc != kWrite) { uint32_t c = P->load[src][dst][x]; if (!c) continue; coef += c; }
              if (acc != kRead) { uint32_t c = P->store[dst][src][x]; if (!c) continue; coef += c; }
              if (cv) coef += P->convert;
              const uint32_t combo2 = combo - (src - dst) * P->lvpow[i];
              uint32_t v2 = v;
              if (x) v2 ^= 1u << P->lay_bit[i];
              if (cv) v2 &= ~(1u << P->dt_bit[i]);
              const uint32_t m2 = c_mask[combo2];
              uint64_t sub = kInf;
              if ((m2 >> v2) & 1u) sub = t_cost[c_base[combo2] + __popc(m2 & ((1u << v2) - 1u))];
              const uint32_t id = P->move_base + ((i * (NL - 1) + dst) * 2 + x) * 2 + cv;
              consider(e, affine(e, 1, sub, mul_checked(e, coef, S.numel[i])), id);
            }
      }

      // C, D. tiles and bufferize, evaluated above
      const uint64_t tb = t_cost[q];
      if (tb < e.best) { e.best = tb; e.arg = sp >> 16; }

      const uint32_t off = (combo * npass + pass) * V + v;
      t_cost[q] = e.best;
      cost[group + off] = e.best;
      arg[group + off] = (uint16_t)e.arg;
      tot.n += e.n;
      tot.ovf |= e.ovf;
    }
    __syncthreads();
  }

  // ---- 5. counters (integer sums: order-independent) ----
  uint32_t n = tot.n;
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) n += __shfl_down(n, d, 64);
  if (lane_id() == 0 && n) atomicAdd(&ctr->n_rewrites, (unsigned long long)n);
  if (tid == 0 && n_task) atomicAdd(&ctr->n_admissible, (unsigned long long)n_task);
  if (tot.ovf) atomicOr(&ctr->overflow, 1u);
}

void launch_fill_level(int block, const DevParams* P, const uint32_t* level_shapes, uint32_t n_units,
                       uint64_t* cost, uint16_t* arg, Counters* ctr, size_t lds_bytes, hipStream_t stream) {
  if (n_units == 0) return;
  if (block == 64)
    hipLaunchKernelGGL(fill_level_kernel<64>, dim3(n_units), dim3(64), lds_bytes, stream, P, level_shapes, n_units, cost, arg, ctr);
  else
    hipLaunchKernelGGL(fill_level_kernel<256>, dim3(n_units), dim3(256), lds_bytes, stream, P, level_shapes, n_units, cost, arg, ctr);
}

}  // namespace mrl
