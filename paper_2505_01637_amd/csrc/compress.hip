// Spatial compression of the dense table into boxes.
//
// Paper, Section 4.1 / Figure 2: every entry starts as a unit rectangle; equal
// adjacent rectangles are merged when their union fills its bounding box.  The
// decision and the volume-normalised cost are compressed separately.
//
// The merge is made canonical by fixing an axis order; along each axis in
// turn, boxes that agree in value and in their extent on every other axis are
// chained when one starts where the previous one ends.
//
// GPU formulation.
//   pass 0  (dense, first axis a0): lanes walk lines of cells along a0 and flag
//           the cells where the value changes (cells whose operands do not fit
//           their levels hold (INF, NONE) by construction and are not read: a
//           bit map from the fill says which cells those are).  Consecutive
//           lanes hold consecutive cells, so the flags of 64 cells are one
//           ballot = one word of a bit mask in table order; the same flags are
//           also kept line-major.  A prefix sum of the popcounts gives every
//           run (= box) its index in table order.
//   pass a  (on boxes): a box looks at the cell just past its end on axis a.
//           If that cell is the low corner of a live box of the same value and
//           the same extents on all other axes, the two are linked; heads of
//           chains then absorb their chain.  The low corner of a box is found
//           in O(1) through the bit mask and the prefix sums.  After the first
//           of these passes the live boxes move to dense arrays; the trailing
//           passes over the innermost bit axes are one kernel.
//   final   live boxes are compacted in index order = sorted by low corner.
#include <hip/hip_runtime.h>
#include "dev_params.h"
#include "compress.h"

namespace mrl {

// ---------------------------------------------------------------- value equality
// Normalised costs c1/vol1 and c2/vol2 where the volumes differ only by the
// factor s1 : s2 of one size axis.  Exact: 128-bit cross multiplication.
__device__ __forceinline__ bool norm_equal(uint64_t c1, uint32_t s1, uint64_t c2, uint32_t s2) {
  if (c1 == kInf || c2 == kInf) return c1 == c2;
  uint64_t a_lo = c1 * s2, a_hi = __umul64hi(c1, s2);
  uint64_t b_lo = c2 * s1, b_hi = __umul64hi(c2, s1);
  return a_lo == b_lo && a_hi == b_hi;
}

// ---------------------------------------------------------------- pass 0
constexpr uint32_t kCellWords = 8;         // 64-cell words a wave of the lane-per-cell kernels takes (a wave per word is mostly wave launch)

// A line = all cells sharing every coordinate but a0.  General form (any stride): one lane per
// cell compares its value with the cell before it on the line; a wave covers one 64-cell word of
// the table-order masks and writes it whole (ballots: no atomics, no zeroing).
__global__ __launch_bounds__(256) void head_flags_kernel(Geo g, uint32_t a0,
                                                         const uint64_t* __restrict__ cost,
                                                         const uint16_t* __restrict__ arg,
                                                         const uint32_t* __restrict__ fitmap,
                                                         const uint32_t* __restrict__ axis_sizes,
                                                         unsigned long long* __restrict__ maskD,
                                                         unsigned long long* __restrict__ maskC) {
  const uint32_t s0 = g.stride[a0], e0 = g.ext[a0];
  const uint32_t word0 = (blockIdx.x * 4u + (threadIdx.x >> 6)) * kCellWords;     // a wave takes kCellWords words
#pragma unroll
  for (uint32_t w = 0; w < kCellWords; w++) {
    const uint32_t cell = (word0 + w) * 64u + (threadIdx.x & 63u);
    const bool active = cell < g.n;
    bool hd = false, hc = false;
    if (active) {
      const uint32_t j = (cell / s0) % e0;
      const bool fits = (fitmap[cell >> 5] >> (cell & 31u)) & 1u;     // cells that cannot fit hold (INF, NONE): not read
      const uint64_t c = fits ? cost[cell] : kInf;
      const uint32_t a = fits ? arg[cell] : kNone;
      hd = hc = true;
      if (j > 0) {
        const uint32_t p = cell - s0;
        const bool pfits = (fitmap[p >> 5] >> (p & 31u)) & 1u;
        const uint64_t pc = pfits ? cost[p] : kInf;
        const uint32_t pa = pfits ? arg[p] : kNone;
        const uint32_t sz = axis_sizes ? axis_sizes[j] : 1u, ps = axis_sizes ? axis_sizes[j - 1] : 1u;
        hd = a != pa;
        hc = !norm_equal(c, sz, pc, ps);
      }
    }
    const unsigned long long bd = __ballot(hd), bc = __ballot(hc);
    if ((threadIdx.x & 63u) == 0 && active) {
      maskD[cell >> 6] = bd;
      maskC[cell >> 6] = bc;
    }
  }
}

// The same for lines whose stride is a multiple of 64 cells (every table with at least 64
// entries per shape): the 64 lanes of a wave then stand on 64 consecutive cells at every step, so
// one 64-bit word of the fit bit map covers the step and one ballot is one word of the mask.  A
// step's cells lie far from the previous step's, so every read is a trip to HBM; to have few of
// them wait for each other, the fit words of up to 64 steps are fetched by one gather (lane t
// holds step t's word), and the values of 8 steps are fetched together before they are compared.
constexpr int kHeadBatch = 8;
constexpr uint32_t kHeadSpread = 32;

__device__ __forceinline__ unsigned long long readlane64(unsigned long long v, uint32_t lane) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, (int)lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), (int)lane);
  return (unsigned long long)hi << 32 | lo;
}

__global__ __launch_bounds__(256) void head_flags_wave_kernel(Geo g, uint32_t a0,
                                                              const uint64_t* __restrict__ cost,
                                                              const uint16_t* __restrict__ arg,
                                                              const unsigned long long* __restrict__ fitmap,
                                                              const uint32_t* __restrict__ axis_sizes,
                                                              unsigned long long* __restrict__ maskD,
                                                              unsigned long long* __restrict__ maskC,
                                                              unsigned long long* __restrict__ lineD,
                                                              unsigned long long* __restrict__ lineC) {
  const uint32_t s0 = g.stride[a0], e0 = g.ext[a0];
  const uint32_t n_lines = g.n / e0;                  // a multiple of 64, as s0 is
  const uint32_t lane = threadIdx.x & 63u;
  // Workgroups that run at the same time work on kHeadSpread distant parts of the table (measured:
  // the pass is a quarter faster than with neighbours side by side); four consecutive workgroups
  // stay together, as their 16 waves fill whole 128-byte lines of the masks.  The grid is padded
  // to a multiple of 4 * kHeadSpread workgroups.
  const uint32_t nch = gridDim.x >> 2, ch = blockIdx.x >> 2;
  const uint32_t blk = ((ch % kHeadSpread) * (nch / kHeadSpread) + ch / kHeadSpread) << 2 | (blockIdx.x & 3u);
  const uint32_t q = blk * 256u + threadIdx.x, q0 = q - lane;
  if (q0 >= n_lines) return;                          // the whole wave
  const uint32_t hi0 = q0 / s0;
  const uint32_t base0 = hi0 * s0 * e0 + (q0 - hi0 * s0);      // lane 0's first cell: a multiple of 64
  uint64_t pc = 0; uint32_t pa = 0, ps = 1;
  // a chunk = up to 64 steps: lane t fetches the fit word of step j0 + t, and in the end stores
  // the two mask words of that step; a line's own flags of the chunk are one word per lane
  for (uint32_t j0 = 0; j0 < e0; j0 += 64) {
    const uint32_t jt = j0 + lane;
    const unsigned long long words = jt < e0 ? fitmap[(base0 + jt * s0) >> 6] : 0ull;
    const uint32_t sizes = (axis_sizes && jt < e0) ? axis_sizes[jt] : 1u;
    const uint32_t n_here = e0 - j0 < 64u ? e0 - j0 : 64u;
    unsigned long long od = 0, oc = 0, wd = 0, wc = 0;
    // steps [0, n_live) hold the cells that fit; past them every cell holds (INF, NONE), so that
    // only step n_live can still start a run
    const unsigned long long live = __ballot(words != 0);
    const uint32_t n_live = live ? 64u - (uint32_t)__builtin_clzll(live) : 0u;
    for (uint32_t u0 = 0; u0 < n_live; u0 += kHeadBatch) {
      uint64_t c[kHeadBatch];
      uint32_t a[kHeadBatch];
#pragma unroll
      for (int u = 0; u < kHeadBatch; u++) {
        const uint32_t t = u0 + u < n_live ? u0 + u : n_live - 1;
        const bool fits = (readlane64(words, t) >> lane) & 1ull;
        const uint32_t cell = base0 + lane + (j0 + t) * s0;
        c[u] = fits ? cost[cell] : kInf;
        a[u] = fits ? (uint32_t)arg[cell] : kNone;
      }
#pragma unroll
      for (int u = 0; u < kHeadBatch; u++) {
        if (u0 + u < n_live) {
          const uint32_t t = u0 + u, j = j0 + t;
          const uint32_t sz = (uint32_t)__builtin_amdgcn_readlane((int)sizes, (int)t);
          const bool hd = j == 0 || a[u] != pa;
          const bool hc = j == 0 || !norm_equal(c[u], sz, pc, ps);
          pc = c[u]; pa = a[u]; ps = sz;
          const unsigned long long bd = __ballot(hd), bc = __ballot(hc);
          if (lane == t) { od = bd; oc = bc; }
          wd |= (unsigned long long)hd << t;
          wc |= (unsigned long long)hc << t;
        }
      }
    }
    if (n_live < n_here) {
      const uint32_t t = n_live;
      const bool hd = j0 + t == 0 || pa != kNone, hc = j0 + t == 0 || pc != kInf;
      const unsigned long long bd = __ballot(hd), bc = __ballot(hc);
      if (lane == t) { od = bd; oc = bc; }
      wd |= (unsigned long long)hd << t;
      wc |= (unsigned long long)hc << t;
      pc = kInf; pa = kNone;
      ps = (uint32_t)__builtin_amdgcn_readlane((int)sizes, (int)(n_here - 1));
    }
    if (jt < e0) {
      const uint32_t w = (base0 + jt * s0) >> 6;
      maskD[w] = od;
      maskC[w] = oc;
    }
    lineD[(size_t)(j0 >> 6) * n_lines + q] = wd;
    lineC[(size_t)(j0 >> 6) * n_lines + q] = wc;
  }
}

// alive[b]: 0 once box b has been merged into another; else kLive | the stamp of the last pass in
// which a box linked to it (one byte for both: a live box stays live when it is linked to, so the
// linking thread can store the whole byte, and a byte less per box is written when the boxes are made).
constexpr uint8_t kLive = 0x80;

// ---------------------------------------------------------------- prefix sums
struct LoadPopc {
  const unsigned long long* p;
  __device__ __forceinline__ uint32_t operator()(uint32_t i) const { return (uint32_t)__popcll(p[i]); }
};
struct LoadFlag {
  const uint8_t* p;
  __device__ __forceinline__ uint32_t operator()(uint32_t i) const { return p[i] ? 1u : 0u; }
};

constexpr uint32_t kScanItems = 8, kScanBlock = 256, kScanTile = kScanItems * kScanBlock;

__device__ __forceinline__ uint32_t block_reduce_256(uint32_t v, uint32_t* sh) {
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) v += __shfl_down(v, d, 64);
  if ((threadIdx.x & 63u) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  uint32_t t = sh[0] + sh[1] + sh[2] + sh[3];
  __syncthreads();
  return t;
}

template <class L>
__global__ __launch_bounds__(256) void scan_tile_sums_kernel(L load, uint32_t n, uint32_t* __restrict__ tile_sum) {
  __shared__ uint32_t sh[4];
  const uint32_t first = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  uint32_t s = 0;
#pragma unroll
  for (uint32_t i = 0; i < kScanItems; i++) if (first + i < n) s += load(first + i);
  const uint32_t t = block_reduce_256(s, sh);
  if (threadIdx.x == 0) tile_sum[blockIdx.x] = t;
}

// One workgroup: exclusive scan of tile_sum in place; the grand total goes to *total.
__global__ __launch_bounds__(256) void scan_top_kernel(uint32_t* __restrict__ tile_sum, uint32_t n_tiles,
                                                       uint32_t* __restrict__ total) {
  __shared__ uint32_t sh[4];
  __shared__ uint32_t carry_sh;
  if (threadIdx.x == 0) carry_sh = 0;
  __syncthreads();
  for (uint32_t base = 0; base < n_tiles; base += 256) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t v = i < n_tiles ? tile_sum[i] : 0;
    uint32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      uint32_t o = __shfl_up(incl, d, 64);
      if ((int)(threadIdx.x & 63u) >= d) incl += o;
    }
    if ((threadIdx.x & 63u) == 63) sh[threadIdx.x >> 6] = incl;
    __syncthreads();
    uint32_t wbase = 0;
    for (uint32_t w = 0; w < (threadIdx.x >> 6); w++) wbase += sh[w];
    const uint32_t carry = carry_sh;
    if (i < n_tiles) tile_sum[i] = carry + wbase + incl - v;
    __syncthreads();
    if (threadIdx.x == 255) carry_sh = carry + wbase + incl;
    __syncthreads();
  }
  if (threadIdx.x == 0) *total = carry_sh;
}

template <class L>
__global__ __launch_bounds__(256) void scan_apply_kernel(L load, uint32_t n, const uint32_t* __restrict__ tile_excl,
                                                         uint32_t* __restrict__ out) {
  __shared__ uint32_t sh[4];
  const uint32_t first = blockIdx.x * kScanTile + threadIdx.x * kScanItems;
  uint32_t v[kScanItems], s = 0;
#pragma unroll
  for (uint32_t i = 0; i < kScanItems; i++) { v[i] = first + i < n ? load(first + i) : 0; s += v[i]; }
  uint32_t incl = s;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t o = __shfl_up(incl, d, 64);
    if ((int)(threadIdx.x & 63u) >= d) incl += o;
  }
  if ((threadIdx.x & 63u) == 63) sh[threadIdx.x >> 6] = incl;
  __syncthreads();
  uint32_t run = tile_excl[blockIdx.x] + incl - s;
  for (uint32_t w = 0; w < (threadIdx.x >> 6); w++) run += sh[w];
#pragma unroll
  for (uint32_t i = 0; i < kScanItems; i++) { if (first + i < n) out[first + i] = run; run += v[i]; }
}

template <class L>
static void exclusive_scan(L load, uint32_t n, uint32_t* tile_tmp, uint32_t* out, uint32_t* total, hipStream_t st) {
  const uint32_t n_tiles = (n + kScanTile - 1) / kScanTile;
  hipLaunchKernelGGL(scan_tile_sums_kernel<L>, dim3(n_tiles), dim3(256), 0, st, load, n, tile_tmp);
  hipLaunchKernelGGL(scan_top_kernel, dim3(1), dim3(256), 0, st, tile_tmp, n_tiles, total);
  hipLaunchKernelGGL(scan_apply_kernel<L>, dim3(n_tiles), dim3(256), 0, st, load, n, tile_tmp, out);
}

void scan_mask_words(const unsigned long long* mask, uint32_t n_words, uint32_t* tile_tmp, uint32_t* prefix,
                     uint32_t* total, hipStream_t st) {
  exclusive_scan(LoadPopc{mask}, n_words, tile_tmp, prefix, total, st);
}

void scan_flags(const uint8_t* flags, uint32_t n, uint32_t* tile_tmp, uint32_t* pos, uint32_t* total, hipStream_t st) {
  exclusive_scan(LoadFlag{flags}, n, tile_tmp, pos, total, st);
}

// The live boxes move to dense arrays, in index order: box b becomes box pos[b].  The old alive[]
// stays as it is: together with pos[] it translates the index a box had after the first pass
// (its rank in the mask) into the new one.
__global__ __launch_bounds__(256) void compact_boxes_kernel(uint32_t n, const uint8_t* __restrict__ alive,
                                                            const uint32_t* __restrict__ pos,
                                                            const uint32_t* __restrict__ bcell,
                                                            const uint4* __restrict__ blen, uint32_t* __restrict__ cell2,
                                                            uint4* __restrict__ len2, uint8_t* __restrict__ alive2) {
  const uint32_t b = blockIdx.x * 256u + threadIdx.x;
  if (b >= n || !alive[b]) return;
  const uint32_t j = pos[b];
  cell2[j] = bcell[b];
  len2[j] = blen[b];
  alive2[j] = kLive;
}

void launch_compact_boxes(uint32_t n, const uint8_t* alive, const uint32_t* pos, const uint32_t* bcell, const void* blen,
                          uint32_t* cell2, void* len2, uint8_t* alive2, hipStream_t st) {
  hipLaunchKernelGGL(compact_boxes_kernel, dim3((n + 255) / 256), dim3(256), 0, st, n, alive, pos, bcell, (const uint4*)blen,
                     cell2, (uint4*)len2, alive2);
}

// ---------------------------------------------------------------- boxes of pass 0

// General form (any stride): one lane per cell; a flagged cell opens the box whose index is its
// rank in the table-order mask (prefix sums), and the box runs to the next flagged cell of the
// line or to the line's end.
__global__ __launch_bounds__(256) void make_boxes_kernel(Geo g, uint32_t a0,
                                                         const unsigned long long* __restrict__ mask,
                                                         const uint32_t* __restrict__ prefix,
                                                         uint32_t* __restrict__ bcell, uint4* __restrict__ blen,
                                                         uint8_t* __restrict__ alive) {
  const uint32_t s0 = g.stride[a0], e0 = g.ext[a0];
  const uint32_t word0 = (blockIdx.x * 4u + (threadIdx.x >> 6)) * kCellWords;
  for (uint32_t wi = 0; wi < kCellWords; wi++) {
    const uint32_t cell = (word0 + wi) * 64u + (threadIdx.x & 63u);
    if (cell >= g.n) return;
    const unsigned long long tm = mask[cell >> 6];
    if (!((tm >> (cell & 63u)) & 1ull)) continue;
    const uint32_t id = prefix[cell >> 6] + (uint32_t)__popcll(tm & ((1ull << (cell & 63u)) - 1ull));
    const uint32_t j = (cell / s0) % e0;
    const uint32_t R = e0 - 1u - j;                       // cells after this one on the line
    uint32_t len = R + 1u;
    if ((s0 & (s0 - 1u)) == 0 && s0 <= 32u) {
      // a power-of-two stride: the line's cells sit at the same bit positions (mod s0) of every
      // word, so the next flagged one is a mask, a count of trailing zeros and a division away
      const unsigned long long P = s0 == 1 ? ~0ull : s0 == 2 ? 0x5555555555555555ull : s0 == 4 ? 0x1111111111111111ull
                                 : s0 == 8 ? 0x0101010101010101ull : s0 == 16 ? 0x0001000100010001ull : 0x0000000100000001ull;
      const uint32_t bit0 = cell & 63u;
      const unsigned long long same = P << (bit0 % s0);
      unsigned long long m = tm & same & ~((2ull << bit0) - 1ull);      // this word: only the cells after this one
      for (uint32_t k = cell >> 6;; m = mask[++k] & same) {
        if (m) {
          const uint32_t t = (k * 64u + (uint32_t)__builtin_ctzll(m) - cell) / s0;
          if (t <= R) len = t;
          break;
        }
        if ((k * 64u + 63u - cell) / s0 >= R) break;      // the line ends inside this word
      }
    } else {
      for (len = 1; len <= R; len++) {
        const uint32_t c2 = cell + len * s0;
        if ((mask[c2 >> 6] >> (c2 & 63u)) & 1ull) break;
      }
    }
    const uint32_t shift = (a0 & 3u) * 8u;
    uint32_t L[4] = {0x01010101u, 0x01010101u, 0x01010101u, 0x01010101u};
    const uint32_t w = (0x01010101u & ~(0xFFu << shift)) | (len << shift);
    L[0] = (a0 >> 2) == 0 ? w : L[0];
    L[1] = (a0 >> 2) == 1 ? w : L[1];
    L[2] = (a0 >> 2) == 2 ? w : L[2];
    L[3] = (a0 >> 2) == 3 ? w : L[3];
    bcell[id] = cell;
    blen[id] = make_uint4(L[0], L[1], L[2], L[3]);
    alive[id] = kLive;
  }
}

// A wave of the word-by-word kernels takes this many consecutive mask words: 64 (one per lane)
// on large tables, few on small ones, which would otherwise occupy a handful of waves for long.
static uint32_t words_per_wave(uint32_t n_words) { return n_words >= (1u << 21) ? 64u : 8u; }

// The same for lines whose stride is a multiple of 64 cells, word by word of the table-order
// mask: a wave takes 64 consecutive words (lane t fetches word t and its prefix sum) and then,
// for every word that flags a cell, stands with its 64 lanes on the word's 64 cells.  These lie
// on 64 consecutive lines at the same step, so the lanes read consecutive words of the line-major
// mask (for the run's end), and the boxes they open have consecutive indices: all of a wave's
// reads and writes are contiguous stretches.
constexpr int kBoxWords = 4;

__global__ __launch_bounds__(256) void make_boxes_wave_kernel(Geo g, uint32_t a0, uint32_t n_words, uint32_t wpw,
                                                              const unsigned long long* __restrict__ mask,
                                                              const uint32_t* __restrict__ prefix,
                                                              const unsigned long long* __restrict__ line,
                                                              const unsigned long long* __restrict__ col, uint32_t a1,
                                                              uint32_t* __restrict__ bcell, uint4* __restrict__ blen,
                                                              uint8_t* __restrict__ alive) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t w0 = (blockIdx.x * 4u + (threadIdx.x >> 6)) * wpw;
  if (w0 >= n_words) return;
  const uint32_t s0 = g.stride[a0], e0 = g.ext[a0], n_lines = g.n / e0, se = s0 * e0;
  const uint32_t shift = (a0 & 3u) * 8u;
  const bool mine = lane < wpw && w0 + lane < n_words;
  const unsigned long long mv = mine ? mask[w0 + lane] : 0ull;
  const uint32_t pv = mine ? prefix[w0 + lane] : 0u;
  // kBoxWords words at a time, so that their reads of the line-major mask are in flight together
  unsigned long long todo = __ballot(mv != 0);
  while (todo) {
    uint32_t id[kBoxWords], cell[kBoxWords], j[kBoxWords], q[kBoxWords], c1[kBoxWords];
    bool head[kBoxWords];
    unsigned long long lm[kBoxWords], cw[kBoxWords];
#pragma unroll
    for (int u = 0; u < kBoxWords; u++) {
      const bool any = todo != 0;
      const uint32_t t = any ? (uint32_t)__ffsll((long long)todo) - 1u : 0u;
      todo &= todo - 1;                 // 0 stays 0
      const unsigned long long m = any ? readlane64(mv, t) : 0ull;
      const uint32_t pf = (uint32_t)__builtin_amdgcn_readlane((int)pv, (int)t);
      const uint32_t cell0 = (w0 + t) * 64u;               // the word's first cell; all 64 share the step j
      const uint32_t hi = cell0 / se, rem = cell0 - hi * se;
      j[u] = rem / s0;
      q[u] = hi * s0 + (rem - j[u] * s0) + lane;
      cell[u] = cell0 + lane;
      id[u] = pf + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
      head[u] = (m >> lane) & 1ull;
      lm[u] = head[u] ? line[(size_t)(j[u] >> 6) * n_lines + q[u]] : 0ull;
      cw[u] = 0; c1[u] = 0;
      if (col) {                        // the runs behind this box on a1 that were folded into it
        const uint32_t s1 = g.stride[a1], e1 = g.ext[a1], se1 = s1 * e1;
        const uint32_t hi1 = cell0 / se1, rem1 = cell0 - hi1 * se1;
        c1[u] = rem1 / s1;
        cw[u] = head[u] ? col[(size_t)hi1 * s1 + (rem1 - c1[u] * s1) + lane] : 0ull;
      }
    }
#pragma unroll
    for (int u = 0; u < kBoxWords; u++) {
      if (head[u]) {
        uint32_t end = e0;                                 // the run ends at the line's next flagged cell
        unsigned long long w = lm[u] & ~((2ull << (j[u] & 63u)) - 1ull);
        for (uint32_t k = j[u] >> 6;;) {
          if (w) { end = k * 64u + (uint32_t)__ffsll((long long)w) - 1u; break; }
          if (++k * 64u >= e0) break;
          w = line[(size_t)k * n_lines + q[u]];
        }
        uint32_t L[4] = {0x01010101u, 0x01010101u, 0x01010101u, 0x01010101u};
        const uint32_t lw = (0x01010101u & ~(0xFFu << shift)) | ((end - j[u]) << shift);
        L[0] = (a0 >> 2) == 0 ? lw : L[0];
        L[1] = (a0 >> 2) == 1 ? lw : L[1];
        L[2] = (a0 >> 2) == 2 ? lw : L[2];
        L[3] = (a0 >> 2) == 3 ? lw : L[3];
        if (col) {
          // bit c of the column word: the run at step c was folded into the one before it
          const unsigned long long above = c1[u] >= 63u ? 0ull : cw[u] >> (c1[u] + 1u);
          const uint32_t more = (uint32_t)__ffsll((long long)~above) - 1u;
          const uint32_t add = more << ((a1 & 3u) * 8u);                       // the byte holds 1
          L[0] += (a1 >> 2) == 0 ? add : 0u;
          L[1] += (a1 >> 2) == 1 ? add : 0u;
          L[2] += (a1 >> 2) == 2 ? add : 0u;
          L[3] += (a1 >> 2) == 3 ? add : 0u;
        }
        bcell[id[u]] = cell[u];
        blen[id[u]] = make_uint4(L[0], L[1], L[2], L[3]);
        alive[id[u]] = kLive;
      }
    }
  }
}

// ---------------------------------------------------------------- the second merge axis, on cells
// The first generic pass would link every run of pass 0 to the run one step further on the second
// merge axis a1 when both have the same value and the same extent on a0 (they differ in no other
// extent yet).  For an a1 that lies outside a0, with a stride of whole mask words and at most 64
// steps, this is decided on the cells before any box exists: a run head whose predecessor on a1
// heads an equal run loses its flag and sets the bit of its step in the word of its column (the
// cells that differ only on a1), from which make_boxes reads the length of the chain.  runs = the
// mask of pass 0, mask2 = the heads of boxes, col = one word per column, zero before.
constexpr int kSecondWords = 4;

// first = the line's mask word that holds step j
__device__ __forceinline__ uint32_t run_end(unsigned long long first, const unsigned long long* __restrict__ line,
                                            uint32_t n_lines, uint32_t e0, uint32_t j, uint32_t q) {
  unsigned long long w = first & ~((2ull << (j & 63u)) - 1ull);
  for (uint32_t k = j >> 6;;) {
    if (w) return k * 64u + (uint32_t)__ffsll((long long)w) - 1u;
    if (++k * 64u >= e0) return e0;
    w = line[(size_t)k * n_lines + q];
  }
}

template <bool COST>
__global__ __launch_bounds__(256) void second_axis_kernel(Geo g, uint32_t a0, uint32_t a1, uint32_t n_words, uint32_t wpw,
                                                          const unsigned long long* __restrict__ runs,
                                                          const unsigned long long* __restrict__ line,
                                                          const unsigned long long* __restrict__ fitmap,
                                                          const uint64_t* __restrict__ cost, const uint16_t* __restrict__ arg,
                                                          const uint32_t* __restrict__ axis_sizes,
                                                          unsigned long long* __restrict__ mask2,
                                                          unsigned long long* __restrict__ col) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t w0 = (blockIdx.x * 4u + (threadIdx.x >> 6)) * wpw;
  if (w0 >= n_words) return;
  const uint32_t s0 = g.stride[a0], e0 = g.ext[a0], n_lines = g.n / e0, se = s0 * e0;
  const uint32_t s1 = g.stride[a1], e1 = g.ext[a1], d = s1 >> 6, back = s1 / se * s0, se1 = s1 * e1;
  const bool mine = lane < wpw && w0 + lane < n_words;
  const unsigned long long mv = mine ? runs[w0 + lane] : 0ull;
  unsigned long long out = mv;
  // kSecondWords words at a time, each stage's reads side by side
  unsigned long long todo = __ballot(mv != 0);
  while (todo) {
    uint32_t t[kSecondWords], w[kSecondWords], c1[kSecondWords];
    unsigned long long m[kSecondWords], cand[kSecondWords], fc[kSecondWords], fp[kSecondWords];
#pragma unroll
    for (int u = 0; u < kSecondWords; u++) {
      const bool any = todo != 0;
      t[u] = any ? (uint32_t)__ffsll((long long)todo) - 1u : 0u;
      todo &= todo - 1;                 // 0 stays 0
      m[u] = any ? readlane64(mv, t[u]) : 0ull;
      w[u] = w0 + t[u];
      c1[u] = (w[u] * 64u / s1) % e1;   // the word's 64 cells share it
      const bool has = m[u] != 0 && c1[u] > 0;
      cand[u] = has ? m[u] & runs[w[u] - d] : 0ull;       // the cell before on a1 heads a run as well
      fc[u] = has ? fitmap[w[u]] : 0ull;
      fp[u] = has ? fitmap[w[u] - d] : 0ull;
    }
    bool me[kSecondWords];
    uint64_t vc[kSecondWords], vp[kSecondWords];
#pragma unroll
    for (int u = 0; u < kSecondWords; u++) {
      me[u] = (cand[u] >> lane) & 1ull;
      const uint32_t cell = w[u] * 64u + lane;
      const bool rc = me[u] && ((fc[u] >> lane) & 1ull), rp = me[u] && ((fp[u] >> lane) & 1ull);
      if (COST) {
        vc[u] = rc ? cost[cell] : kInf;
        vp[u] = rp ? cost[cell - s1] : kInf;
      } else {
        vc[u] = rc ? (uint64_t)arg[cell] : (uint64_t)kNone;
        vp[u] = rp ? (uint64_t)arg[cell - s1] : (uint64_t)kNone;
      }
    }
    bool same[kSecondWords];
    uint32_t j[kSecondWords], q[kSecondWords];
    unsigned long long lc[kSecondWords], lp[kSecondWords];
#pragma unroll
    for (int u = 0; u < kSecondWords; u++) {
      if (COST) {
        const uint32_t z1 = (axis_sizes && c1[u]) ? axis_sizes[c1[u] - 1] : 1u, z2 = axis_sizes ? axis_sizes[c1[u]] : 1u;
        same[u] = me[u] && norm_equal(vp[u], z1, vc[u], z2);
      } else {
        same[u] = me[u] && vp[u] == vc[u];
      }
      const uint32_t cell0 = w[u] * 64u, hi = cell0 / se, rem = cell0 - hi * se;
      j[u] = rem / s0;
      q[u] = hi * s0 + (rem - j[u] * s0) + lane;
      const size_t at = (size_t)(j[u] >> 6) * n_lines + q[u];
      lc[u] = same[u] ? line[at] : 0ull;
      lp[u] = same[u] ? line[at - back] : 0ull;
    }
#pragma unroll
    for (int u = 0; u < kSecondWords; u++) {
      if (same[u])        // equal extents on a0: both runs end at the same step
        same[u] = run_end(lc[u], line, n_lines, e0, j[u], q[u]) == run_end(lp[u], line, n_lines, e0, j[u], q[u] - back);
      if (same[u]) {
        const uint32_t cell0 = w[u] * 64u, hi1 = cell0 / se1, rem1 = cell0 - hi1 * se1;
        atomicOr(&col[(size_t)hi1 * s1 + (rem1 - c1[u] * s1) + lane], 1ull << c1[u]);
      }
      const unsigned long long gone = __ballot(same[u]);
      if (m[u] && lane == t[u]) out = m[u] & ~gone;
    }
  }
  if (mine) mask2[w0 + lane] = out;
}

// ---------------------------------------------------------------- pass on axis a
__device__ __forceinline__ uint32_t len_byte(const uint4& L, uint32_t a) {
  const uint32_t w = a < 4 ? L.x : a < 8 ? L.y : a < 12 ? L.z : L.w;
  return (w >> ((a & 3u) * 8)) & 0xFFu;
}

// Every box still has extent 1 on axis a when its pass comes (an axis is merged once).  Most
// boxes differ in value from the cell past their end, so the values are compared first and the
// extents are read only for the few that pass.  block_linked[workgroup] tells the absorb step
// whether any of the workgroup's boxes got a successor.  After the compaction the mask still
// ranks boxes by their old index: old_alive / remap translate it (nullptr before).
template <bool COST>
__global__ __launch_bounds__(256) void link_kernel(Geo g, uint32_t a, uint8_t stamp, uint32_t n_boxes,
                                                   const uint8_t* __restrict__ old_alive,
                                                   const uint32_t* __restrict__ remap,
                                                   const uint32_t* __restrict__ bcell, const uint4* __restrict__ blen,
                                                   uint8_t* alive,
                                                   uint32_t* __restrict__ next, uint32_t* __restrict__ block_linked,
                                                   const unsigned long long* __restrict__ mask,
                                                   const uint32_t* __restrict__ prefix,
                                                   const uint64_t* __restrict__ cost, const uint16_t* __restrict__ arg,
                                                   const uint32_t* __restrict__ axis_sizes) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  const uint32_t b = i < n_boxes ? i : 0u;
  const bool live = i < n_boxes && alive[b];
  uint32_t nxt = 0xFFFFFFFFu;
  if (live) {
    const uint32_t cell = bcell[b];
    const uint32_t sa = g.stride[a], ea = g.ext[a];
    const uint32_t ca = (cell / sa) % ea;
    if (ca + 1 < ea) {
      const uint32_t s = cell + sa;
      bool same;
      if (COST) {
        const uint32_t s1 = axis_sizes ? axis_sizes[ca] : 1u, s2 = axis_sizes ? axis_sizes[ca + 1] : 1u;
        same = norm_equal(cost[cell], s1, cost[s], s2);
      } else {
        same = arg[cell] == arg[s];
      }
      if (same) {
        const unsigned long long m = mask[s >> 6];
        if ((m >> (s & 63u)) & 1ull) {
          uint32_t o = prefix[s >> 6] + (uint32_t)__popcll(m & ((1ull << (s & 63u)) - 1ull));
          bool there = true;
          if (remap) { there = old_alive[o]; o = there ? remap[o] : 0u; }
          if (there && alive[o]) {
            const uint4 L = blen[b], M = blen[o];     // equal on a as well: both 1
            if (L.x == M.x && L.y == M.y && L.z == M.z && L.w == M.w) {
              nxt = o;
              alive[o] = kLive | stamp;
            }
          }
        }
      }
    }
    next[b] = nxt;
  }
  const int any = __syncthreads_or(nxt != 0xFFFFFFFFu);
  if (threadIdx.x == 0) block_linked[blockIdx.x] = (uint32_t)any;
}

__global__ __launch_bounds__(256) void absorb_kernel(uint32_t a, uint8_t stamp, uint32_t n_boxes,
                                                     uint8_t* __restrict__ blen_bytes,
                                                     uint8_t* alive,
                                                     const uint32_t* __restrict__ next,
                                                     const uint32_t* __restrict__ block_linked) {
  if (!block_linked[blockIdx.x]) return;       // no box of this workgroup got a successor: no chain starts here
  const uint32_t b = blockIdx.x * 256u + threadIdx.x;
  if (b >= n_boxes) return;
  uint32_t s = next[b];
  if (s == 0xFFFFFFFFu || !alive[b] || alive[b] == (kLive | stamp)) return;   // only heads of chains of two or more
  uint32_t tot = blen_bytes[(size_t)b * 16 + a];
  for (; s != 0xFFFFFFFFu; s = next[s]) {
    tot += blen_bytes[(size_t)s * 16 + a];
    alive[s] = 0;
  }
  blen_bytes[(size_t)b * 16 + a] = (uint8_t)tot;
}

void launch_head_flags(const Geo& g, uint32_t a0, const uint64_t* cost, const uint16_t* arg, const uint32_t* fitmap,
                       const uint32_t* axis_sizes,
                       unsigned long long* maskD, unsigned long long* maskC, unsigned long long* lineD,
                       unsigned long long* lineC, hipStream_t st) {
  const uint32_t n_lines = g.n / g.ext[a0];
  const uint32_t blocks = (n_lines + 255) / 256;
  if (g.stride[a0] % 64 == 0)
    hipLaunchKernelGGL(head_flags_wave_kernel, dim3((blocks + 4 * kHeadSpread - 1) / (4 * kHeadSpread) * (4 * kHeadSpread)), dim3(256), 0, st, g, a0, cost, arg,
                       (const unsigned long long*)fitmap, axis_sizes, maskD, maskC, lineD, lineC);
  else
    hipLaunchKernelGGL(head_flags_kernel, dim3((g.n + 256 * kCellWords - 1) / (256 * kCellWords)), dim3(256), 0, st, g, a0, cost, arg, fitmap, axis_sizes,
                       maskD, maskC);
}

void launch_second_axis(const Geo& g, uint32_t a0, uint32_t a1, bool is_cost, const unsigned long long* runs,
                        const unsigned long long* line, const uint32_t* fitmap, const uint64_t* cost, const uint16_t* arg,
                        const uint32_t* axis_sizes, unsigned long long* mask2, unsigned long long* col, hipStream_t st) {
  const uint32_t n_words = g.n / 64;
  const uint32_t wpw = words_per_wave(n_words);
  const dim3 grid((n_words + 4 * wpw - 1) / (4 * wpw));
  if (is_cost)
    hipLaunchKernelGGL(second_axis_kernel<true>, grid, dim3(256), 0, st, g, a0, a1, n_words, wpw, runs, line,
                       (const unsigned long long*)fitmap, cost, arg, axis_sizes, mask2, col);
  else
    hipLaunchKernelGGL(second_axis_kernel<false>, grid, dim3(256), 0, st, g, a0, a1, n_words, wpw, runs, line,
                       (const unsigned long long*)fitmap, cost, arg, axis_sizes, mask2, col);
}

void launch_make_boxes(const Geo& g, uint32_t a0, const unsigned long long* mask, const uint32_t* prefix,
                       const unsigned long long* line, const unsigned long long* col, uint32_t a1, uint32_t* bcell,
                       void* blen, uint8_t* alive, hipStream_t st) {
  if (g.stride[a0] % 64 == 0) {
    const uint32_t n_words = g.n / 64;
    const uint32_t wpw = words_per_wave(n_words);
    hipLaunchKernelGGL(make_boxes_wave_kernel, dim3((n_words + 4 * wpw - 1) / (4 * wpw)), dim3(256), 0, st, g, a0, n_words, wpw, mask, prefix,
                       line, col, a1, bcell, (uint4*)blen, alive);
  } else {
    hipLaunchKernelGGL(make_boxes_kernel, dim3((g.n + 256 * kCellWords - 1) / (256 * kCellWords)), dim3(256), 0, st, g, a0, mask, prefix, bcell,
                       (uint4*)blen, alive);
  }
}

void launch_axis_pass(const Geo& g, uint32_t a, uint8_t stamp, bool is_cost, uint32_t n_boxes, const uint8_t* old_alive,
                      const uint32_t* remap, const uint32_t* bcell, void* blen, uint8_t* alive, uint32_t* next,
                      uint32_t* block_linked, const unsigned long long* mask, const uint32_t* prefix, const uint64_t* cost,
                      const uint16_t* arg, const uint32_t* axis_sizes, hipStream_t st) {
  const uint32_t blocks = (n_boxes + 255) / 256;
  if (is_cost)
    hipLaunchKernelGGL(link_kernel<true>, dim3(blocks), dim3(256), 0, st, g, a, stamp, n_boxes, old_alive, remap, bcell,
                       (const uint4*)blen, alive, next, block_linked, mask, prefix, cost, arg, axis_sizes);
  else
    hipLaunchKernelGGL(link_kernel<false>, dim3(blocks), dim3(256), 0, st, g, a, stamp, n_boxes, old_alive, remap, bcell,
                       (const uint4*)blen, alive, next, block_linked, mask, prefix, cost, arg, axis_sizes);
  hipLaunchKernelGGL(absorb_kernel, dim3(blocks), dim3(256), 0, st, a, stamp, n_boxes, (uint8_t*)blen, alive, next,
                     block_linked);
}

// ---------------------------------------------------------------- the last passes, in one
// The merge order ends with the axes of the layout and dtype bits, which are also the innermost
// coordinates: extent 2 and a stride of at most 32 cells, so a box and the one it could merge
// with on such an axis have their low corners in the same 64-cell word of the mask, and no chain
// is longer than two.  A wave stands with its lanes on the cells of a word, holds the live boxes
// that start there in registers, and runs all those passes with lane exchanges: one read and at
// most one write of every box instead of one per pass.
constexpr int kTailWords = 4;

template <bool COST>
__global__ __launch_bounds__(256) void tail_pairs_kernel(TailAxes T, uint32_t n_words, uint32_t wpw,
                                                         const unsigned long long* __restrict__ mask,
                                                         const uint32_t* __restrict__ prefix,
                                                         const uint8_t* __restrict__ old_alive,
                                                         const uint32_t* __restrict__ remap, uint4* __restrict__ blen,
                                                         uint8_t* __restrict__ alive, const uint64_t* __restrict__ cost,
                                                         const uint16_t* __restrict__ arg) {
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t w0 = (blockIdx.x * 4u + (threadIdx.x >> 6)) * wpw;
  if (w0 >= n_words) return;
  const bool mine = lane < wpw && w0 + lane < n_words;
  const unsigned long long mv = mine ? mask[w0 + lane] : 0ull;
  const uint32_t pv = mine ? prefix[w0 + lane] : 0u;
  // kTailWords words at a time, their reads side by side: every read is a trip to memory, and a
  // word needs four of them in a row (old alive, new index, live, extents and value)
  unsigned long long todo = __ballot(mv != 0);
  while (todo) {
    uint32_t id[kTailWords], cell[kTailWords];
    bool live[kTailWords];
#pragma unroll
    for (int u = 0; u < kTailWords; u++) {
      const bool any = todo != 0;
      const uint32_t t = any ? (uint32_t)__ffsll((long long)todo) - 1u : 0u;
      todo &= todo - 1;                 // 0 stays 0
      const unsigned long long m = any ? readlane64(mv, t) : 0ull;
      const uint32_t pf = (uint32_t)__builtin_amdgcn_readlane((int)pv, (int)t);
      cell[u] = (w0 + t) * 64u + lane;
      id[u] = pf + (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
      live[u] = (m >> lane) & 1ull;
    }
    if (remap) {                       // the mask ranks boxes by the index they had before the compaction
#pragma unroll
      for (int u = 0; u < kTailWords; u++) live[u] = live[u] && old_alive[id[u]];
#pragma unroll
      for (int u = 0; u < kTailWords; u++) id[u] = live[u] ? remap[id[u]] : 0u;
    }
#pragma unroll
    for (int u = 0; u < kTailWords; u++) live[u] = live[u] && alive[id[u]];
    uint4 L[kTailWords];
    uint64_t v[kTailWords];
#pragma unroll
    for (int u = 0; u < kTailWords; u++) {
      L[u] = live[u] ? blen[id[u]] : make_uint4(0, 0, 0, 0);
      // the two boxes of a pair start in the same shape, so equal normalised costs = equal costs
      v[u] = 0;
      if (live[u]) v[u] = COST ? cost[cell[u]] : (uint64_t)arg[cell[u]];
    }
#pragma unroll
    for (int u = 0; u < kTailWords; u++) {
      if (!__any(live[u])) continue;
      bool changed = false, died = false;
      for (uint32_t k = 0; k < T.n; k++) {
        const uint32_t st = T.stride[k], a = T.axis[k];
        const int p_live = __shfl_down((int)live[u], st, 64);
        const uint32_t p_lo = __shfl_down((uint32_t)v[u], st, 64), p_hi = __shfl_down((uint32_t)(v[u] >> 32), st, 64);
        const uint32_t px = __shfl_down(L[u].x, st, 64), py = __shfl_down(L[u].y, st, 64);
        const uint32_t pz = __shfl_down(L[u].z, st, 64), pw = __shfl_down(L[u].w, st, 64);
        const bool low = (lane & st) == 0;             // coordinate 0 on this axis: lane + st is in the same word
        const bool merge = low && live[u] && p_live && (uint32_t)v[u] == p_lo && (uint32_t)(v[u] >> 32) == p_hi &&
                           L[u].x == px && L[u].y == py && L[u].z == pz && L[u].w == pw;
        if (merge) {
          const uint32_t one = 1u << ((a & 3u) * 8u);
          L[u].x += (a >> 2) == 0 ? one : 0u;
          L[u].y += (a >> 2) == 1 ? one : 0u;
          L[u].z += (a >> 2) == 2 ? one : 0u;
          L[u].w += (a >> 2) == 3 ? one : 0u;
          changed = true;
        }
        const int absorbed = __shfl_up((int)merge, st, 64);
        if (!low && absorbed) { live[u] = false; died = true; }
      }
      if (changed) blen[id[u]] = L[u];
      if (died) alive[id[u]] = 0;
    }
  }
}

void launch_tail_pairs(const TailAxes& T, bool is_cost, uint32_t n_words, const unsigned long long* mask,
                       const uint32_t* prefix, const uint8_t* old_alive, const uint32_t* remap, void* blen, uint8_t* alive,
                       const uint64_t* cost, const uint16_t* arg, hipStream_t st) {
  const uint32_t wpw = words_per_wave(n_words), blocks = (n_words + 4 * wpw - 1) / (4 * wpw);
  if (is_cost)
    hipLaunchKernelGGL(tail_pairs_kernel<true>, dim3(blocks), dim3(256), 0, st, T, n_words, wpw, mask, prefix, old_alive, remap,
                       (uint4*)blen, alive, cost, arg);
  else
    hipLaunchKernelGGL(tail_pairs_kernel<false>, dim3(blocks), dim3(256), 0, st, T, n_words, wpw, mask, prefix, old_alive, remap,
                       (uint4*)blen, alive, cost, arg);
}

// ---------------------------------------------------------------- final lists
// Binary gcd (shifts and subtractions: a 64-bit remainder is a long software routine here).
__device__ __forceinline__ uint64_t gcd_u64(uint64_t a, uint64_t b) {
  if (a == 0) return b;
  if (b == 0) return a;
  const int shift = __builtin_ctzll(a | b);
  a >>= __builtin_ctzll(a);
  do {
    b >>= __builtin_ctzll(b);
    if (a > b) { const uint64_t t = a; a = b; b = t; }
    b -= a;
  } while (b);
  return a << shift;
}

template <bool COST>
__global__ __launch_bounds__(256) void emit_kernel(Geo g, const DevParams* __restrict__ P,
                                                   uint32_t n_boxes,
                                                   const uint32_t* __restrict__ bcell, const uint4* __restrict__ blen,
                                                   const uint8_t* __restrict__ alive, const uint32_t* __restrict__ pos,
                                                   const uint64_t* __restrict__ cost, const uint16_t* __restrict__ arg,
                                                   uint32_t* __restrict__ fcell, uint4* __restrict__ flen,
                                                   uint64_t* __restrict__ fv0, uint64_t* __restrict__ fv1) {
  const uint32_t b = blockIdx.x * 256u + threadIdx.x;
  if (b >= n_boxes || !alive[b]) return;
  const uint32_t o = pos[b], cell = bcell[b];
  fcell[o] = cell;
  flen[o] = blen[b];
  if (COST) {
    const uint64_t c = cost[cell];
    if (c == kInf) { fv0[o] = kInf; fv1[o] = 0; }
    else {
      uint64_t vol = 1;
#pragma unroll
      for (int d = 0; d < 4; d++) vol *= P->sizes[d][(cell / g.stride[d]) % g.ext[d]];
      const uint64_t q = gcd_u64(c, vol);
      fv0[o] = c / q; fv1[o] = vol / q;
    }
  } else {
    fv0[o] = arg[cell]; fv1[o] = 0;
  }
}

void launch_emit(const Geo& g, const DevParams* P, bool is_cost, uint32_t n_boxes, const uint32_t* bcell,
                 const void* blen,
                 const uint8_t* alive, const uint32_t* pos, const uint64_t* cost, const uint16_t* arg, uint32_t* fcell,
                 void* flen, uint64_t* fv0, uint64_t* fv1, hipStream_t st) {
  const uint32_t blocks = (n_boxes + 255) / 256;
  if (is_cost)
    hipLaunchKernelGGL(emit_kernel<true>, dim3(blocks), dim3(256), 0, st, g, P, n_boxes, bcell, (const uint4*)blen,
                       alive, pos, cost, arg, fcell, (uint4*)flen, fv0, fv1);
  else
    hipLaunchKernelGGL(emit_kernel<false>, dim3(blocks), dim3(256), 0, st, g, P, n_boxes, bcell, (const uint4*)blen,
                       alive, pos, cost, arg, fcell, (uint4*)flen, fv0, fv1);
}

// ---------------------------------------------------------------- query
__global__ __launch_bounds__(256) void gather_kernel(const uint64_t* __restrict__ idx, uint32_t n,
                                                     const uint64_t* __restrict__ cost, const uint16_t* __restrict__ arg,
                                                     uint64_t* __restrict__ cost_out, uint16_t* __restrict__ arg_out) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= n) return;
  cost_out[i] = cost[idx[i]];
  arg_out[i] = arg[idx[i]];
}

void launch_gather(const uint64_t* idx, uint32_t n, const uint64_t* cost, const uint16_t* arg, uint64_t* cost_out,
                   uint16_t* arg_out, hipStream_t st) {
  hipLaunchKernelGGL(gather_kernel, dim3((n + 255) / 256), dim3(256), 0, st, idx, n, cost, arg, cost_out, arg_out);
}

__global__ __launch_bounds__(256) void zero_words_kernel(unsigned long long* p, uint32_t n) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < n) p[i] = 0;
}

void launch_zero_words(unsigned long long* p, uint32_t n, hipStream_t st) {
  if (n) hipLaunchKernelGGL(zero_words_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n);
}

}  // namespace mrl
