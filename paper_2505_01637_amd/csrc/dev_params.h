// Internal: lattice geometry and target tables as the kernels see them.
// One DevParams lives in device memory per solved table; every field is
// uniform across a workgroup, so reads compile to scalar loads (which is why
// even the small fields are 32 bits wide: there is no scalar byte load).
#pragma once
#include <stdint.h>
#include <hip/hip_runtime.h>

namespace mrl {

constexpr uint64_t kInf = UINT64_MAX;
constexpr uint32_t kNone = 0xFFFFu;
constexpr uint64_t kLimit = 1ull << 62;      // finite costs stay below this
constexpr int kMaxSizes = 256;
constexpr int kMaxCombo = 256;               // n_levels ^ n_operands
constexpr int kMaxRanks = 16;
constexpr uint32_t kNoBit = 0xFF;            // "this operand has no such coordinate"

enum : uint32_t { kKindM = 0, kKindE = 1, kKindF = 2, kKindV = 3,     // V: Move Specs (two tensors: source, destination)
                  kKindR = 4 };                                         // R: ReLU alone (in, out); the bias add alone is kKindE
enum : uint32_t { kRead = 0, kRmw = 1, kWrite = 2 };

// One tile rewrite of a (dim, size index): the index of the smaller size and the trip count.
struct TileEntry {
  uint32_t jt;
  uint32_t trips;
};

// A level assignment of the operands is handled as a "pack": 2 bits per operand,
// operand 0 in the highest field.  pack <-> combo (the mixed-radix index used in
// table offsets) are both kept because offsets need the latter.
struct DevParams {
  // ---- geometry ----
  uint32_t kind, nops, nlv, NL;
  uint32_t npass;            // values of the passive level axis (FUSED: intermediate), else 1
  uint32_t ncombo;           // NL^nops: level assignments of the operands
  uint32_t nlay, ndt, V;     // layout bits, dtype bits, V = 2^(nlay+ndt) variants per combo
  uint32_t log2V;            // V = 1 << log2V
  uint32_t G;                // entries per shape = ncombo * npass * V
  uint32_t nsz[4];
  uint32_t shape_stride[4];  // in shapes
  uint32_t sizes[4][kMaxSizes];
  uint32_t tile_off[4][kMaxSizes + 1];   // CSR into tiles, per (dim, size index)
  const TileEntry* tiles;    // device
  uint32_t tile_dim_ok[4];   // which dims this kind may tile
  uint32_t lay_bit[5];       // bit position inside the variant index, kNoBit = no coordinate
  uint32_t lay_w[5];         // bits of the layout field: 1 (row-/column-major), 2 (also packed and shuffled strips)
  uint32_t dt_bit[5];
  uint32_t base_bf16[5];
  uint32_t access[5];
  uint32_t pack_shift[4];    // bit position of operand i's level inside a pack
  uint32_t lvpow[5];         // combo stride of operand i
  // ---- target ----
  uint64_t cap[4];
  uint32_t convert, zero[4], s;
  uint32_t nmk, mk_kind[8], mk_lanes[8];
  uint64_t mk_cost[8];
  // Move coefficient per element, [operand][src][dst][same|transposed]; load and/or store
  // according to how the operand is accessed; 0 = the Move does not exist.
  uint32_t mcoef[4][4][4][2];
  uint32_t can_convert[4];   // operand may take a converting Move (has a dtype bit and is read-only)
  // per (pack, variant): bit j set = the level/layout/dtype part of microkernel j's predicate holds
  const uint8_t* mk_entry;   // device, [256][V]
  // ---- rewrite ids ----
  uint32_t move_base, tile_base, buf_id, maxs;
  // ---- parallel loops (a Matmul whose serial-only flag is off; kind stays kKindM) ----
  uint32_t par;              // 1: also evaluate parallel loops over b, m, n; their bodies are read from costM
  uint32_t par_base;         // first id of the parallel loops: par_base + dim * maxs + index of the tile size
  uint32_t threads, sync;    // rounds = ceil(trips / threads); constant added per parallel loop
  // ---- operand-level combos ordered by rank (sum of operand levels) ----
  uint32_t nranks;
  uint32_t rank_off[kMaxRanks + 2];
  // per rank-major position: pack | (operands resident in level l, one nibble per level) << 8
  // | (r + 1) << 24 at the first position of rank r
  uint32_t pos_info[kMaxCombo];
  // ---- memory bounds as coordinates (a Matmul lattice whose Specs carry a bound per level of
  // finite capacity; kind stays kKindM).  Bound index q stands for 0 bytes (q = 0) or 2^(q-1).
  uint32_t bounded;          // 1: G = ncombo * Q * V, entry = (combo * Q + bound vector) * V + variant
  uint32_t nlim, Q;          // number of bound axes; Q = product of their extents
  uint32_t lim_nq[4];        // extent of bound axis a
  uint32_t lim_stride[4];    // its stride inside the bound vector's index (first axis slowest)
  uint32_t lim_of_level[4];  // bound axis of memory level l, kNoBit if the level is unbounded
  // ---- Move Specs (kind kKindV) and the Matmul whose Moves are Move Specs (moves = 1, kind kKindM) ----
  // A Move lattice keeps its four abstract-value axes (contiguousness and aligned flag of source and
  // destination) where a bounded lattice keeps its bounds: nlim = 4, lim_nq = {3, 2, 3, 2}.
  uint32_t gather;           // 1: filled by the lane-per-Spec kernel (bounded, Move and moves lattices)
  uint32_t moves;            // 1: a Move costs m(src) + m(dest) + the load / store Move Specs read from costM
  uint32_t weight[4];        // per-level weight of m(t)
  uint32_t line_bytes;
  uint32_t GV, VV, nszV;     // the Move table: entries per shape, variants, number of column sizes
  uint32_t QV, qV_top;       // its abstract vectors per level pair, and the index of (contiguous, aligned) twice
  uint32_t layV[2], dtV[2];  // bit positions of its layout and dtype bits, kNoBit if absent
  uint32_t limV_stride[4];   // strides of its four abstract-value axes inside the abstract vector's index
  // ---- packed layouts (Move lattices and the Matmul whose Moves are Move Specs) ----
  uint32_t strip;            // columns per strip of layouts 2 (packed) and 3 (packed, strips shuffled)
  uint32_t line_mask;        // line_bytes - 1 if line_bytes is a power of two, else 0
  uint32_t xw;               // layout changes a Move id names: 2, or 4 where some operand has a 2-bit layout field
  // ---- tables a FUSED lattice reads (costM also: the serial table a parallel lattice reads) ----
  const uint64_t* costM;
  const uint64_t* costE;
  uint32_t GM, VM, GE, VE, nszE_n;
  uint32_t kM_first, nkM;    // a FUSED lattice's k list starts at entry kM_first of costM's table's, which has nkM entries
  // ---- the composition of two Matmuls (kind stays kKindF: four operands and an intermediate) ----
  // sizes[0] holds p, the dimension the two Matmuls share: lhs m x k, rhs1 k x p, rhs2 p x n, out
  // m x n (accumulated into), intermediate m x p.  Both stages are read from costM.
  uint32_t chain;
  // ---- the bias-add + ReLU with the bufferize between the two (kind stays kKindE) ----
  // One more rewrite per level l of the intermediate (m x n, f32, row-major): the bias-add Spec
  // (in, bias, intermediate) read from costM and the ReLU Spec (intermediate, out) read from costE;
  // GM / VM / layM and GE / VE / layE describe those two tables.  Ids buf_id + l.
  uint32_t split;
  uint32_t layM[3], layE[3]; // layout bit positions in the dependency's variant index
};

// The counts are spread over slots (workgroup index modulo kCtrSlots) and added up by the host:
// atomics of many workgroups on one address serialise (about 10 ns each across the chip), and a
// kernel does not end before its atomics have.
constexpr uint32_t kCtrSlots = 256;
struct Counters {
  unsigned int overflow;
  unsigned int pad;
  unsigned long long n_admissible[kCtrSlots];
  unsigned long long n_rewrites[kCtrSlots];
};

// Layouts (Section 2.4.2): 0 row-major, 1 column-major, 2 packed in strips of s columns, 3 packed
// with shuffled strips.  Physical dimensions of a rows x cols tensor, outermost first: two, or for
// the packed layouts strips, rows, columns of a strip; a tile cut out of one strip (cols < s) is
// the same part of every row of that strip.
// (sizes and the strip are 32-bit by the ABI: divisions stay 32-bit; only products of sizes need 64)
__host__ __device__ inline uint32_t phys_dims(uint32_t layout, uint32_t rows, uint32_t cols, uint32_t s, uint32_t d[3]) {
  if (layout == 0) { d[0] = rows; d[1] = cols; d[2] = 1; return 2; }
  if (layout == 1) { d[0] = cols; d[1] = rows; d[2] = 1; return 2; }
  if (cols >= s) { d[0] = cols / s; d[1] = rows; d[2] = s; }
  else { d[0] = 1; d[1] = rows; d[2] = cols; }
  return 3;
}
__host__ __device__ inline bool layout_fits(uint32_t layout, uint32_t cols, uint32_t s) {
  return layout < 2 || cols % s == 0 || (cols < s && s % cols == 0);
}
// The most inner physical dimensions whose values can be adjacent: the rows of a part of a strip
// lie a strip apart, and the columns of a part of a shuffled strip are no neighbours either.
__host__ __device__ inline uint32_t max_contig(uint32_t layout, uint32_t cols, uint32_t s) {
  if (layout < 2) return 2;
  if (cols >= s) return 3;
  if (layout == 2) return 1;
  return cols == 1 ? 1 : 0;
}

// Section 2.4.3 for a tile of r2 x c2 cut out of a rows x cols tensor in `layout` with element size
// eb: what is known of the tile, given what was known of the tensor.  The tile's values over its
// inner j dimensions are adjacent while the j - 1 innermost are taken whole; it is aligned if the
// tensor was aligned and contiguous in all its dimensions, every suffix product of the tile's
// physical dimensions is a whole number of cache lines, and it is no part of a strip.
// line_mask = line - 1 if the cache line is a power of two (then "multiple of the line" is a mask test), else 0.
__host__ __device__ inline void tile_abstract(uint32_t layout, uint32_t rows, uint32_t cols, uint32_t r2, uint32_t c2, uint32_t eb,
                                              uint32_t strip, uint32_t line, uint32_t line_mask, uint32_t contig, uint32_t aligned,
                                              uint32_t& contig2, uint32_t& aligned2) {
  uint32_t whole[3], part[3];
  const uint32_t nd = phys_dims(layout, rows, cols, strip, whole);
  phys_dims(layout, r2, c2, strip, part);
  uint32_t uncut = 0;
  bool lines_ok = layout < 2 || c2 >= strip;
  uint64_t suffix = eb;
  bool still = true;
#pragma unroll
  for (int q3 = 2; q3 >= 0; q3--) {
    if ((uint32_t)q3 >= nd) continue;
    still = still && part[q3] == whole[q3];
    uncut += still ? 1u : 0u;
    suffix *= part[q3];
    lines_ok = lines_ok && (line_mask || line == 1 ? (suffix & line_mask) == 0 : suffix % line == 0);
  }
  uint32_t keep = 1u + uncut;
  const uint32_t most = max_contig(layout, c2, strip);
  keep = keep < most ? keep : most;
  contig2 = contig < keep ? contig : keep;
  aligned2 = (aligned && contig == nd && lines_ok) ? 1u : 0u;
}

}  // namespace mrl
