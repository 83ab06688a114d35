/*
 * CPU oracle for the memo-table fill and its spatial compression.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded
 * statement of what the method computes, used only to check the HIP library
 * (tests, the smoke check, and the CPU-baseline leg of the benchmark).  It
 * shares no code with the HIP path and the product never calls it.
 *
 * What it follows in the paper:
 *   - Section 4 (Synthesis): top-down search; look the Spec up in the memo
 *     table, else evaluate every applicable rewrite, recurse on the rewrite's
 *     sub-Specs, memoize and return the lowest-cost one.  -> orc_solve()
 *   - Section 3 (Cost Model): c(p) is affine in the sub-program costs:
 *     loop = trips * c(body) + s (parallel: ceil(trips / threads) rounds);
 *     alloc-binding = move cost + c(children);
 *     pipeline/block = sum of children; microkernel = k_p.
 *   - Section 2 (Tiling, Memory Movement, Microkernel Selection) and
 *     Section 2.1 (bufferize of a composition) for the rewrites themselves.
 *   - Section 4.1 (Memoization Database): Specs are points in Z>=0^D;
 *     unit rectangles holding the decision (and, separately, the cost
 *     normalised to the Spec's volume) are merged with adjacent rectangles of
 *     the same value when the union fills its bounding box.  -> orc_merge()
 *
 * Pins (see tests): worked example of Figure 1, brute-force enumeration of all
 * complete schedules on tiny lattices (oracle/brute_force.py, written
 * separately in Python), closed forms, and decompress(merge(x)) == x.
 * The fused three-node lattice (kind 2) follows this build's own reading of
 * Section 2.1; it is pinned by brute force only: "parity unpinned" by the
 * paper beyond the sum rule of Section 3.
 * Kind 3 adds the parallel loops of Section 3; kinds 4, 5, 6 (= kinds 0, 1,
 * 2 with bounds) replace the admissibility test by the per-level memory
 * bounds of Sections 2.2 and 2.4.4, carried as coordinates (expand(), parts
 * B and D).
 * Kind 7 is the lattice of Move Specs (Section 2.2: loads, stores, packing and
 * casts are Specs of their own, implemented by loops over move microkernels
 * such as VectorMove, Section 2), with the contiguousness and alignment
 * abstract values of Section 2.4.3 as coordinates; kind 8 is the Matmul
 * whose Moves are those Specs: an alloc-binding costs m(src) + m(dest)
 * (Section 3, in cache lines) plus its children, the load and store Move
 * Specs among them (Section 2, Memory Movement).
 * Kind 9 is the composition of two Matmuls of Section 2.1, treated like the
 * fused lattice of kind 2: tiles of the output's dimensions, Moves of the
 * four external operands, and one bufferize that splits it into two Matmul
 * Specs around the intermediate.
 * Kinds 10 to 12 take the bias-add + ReLU of kind 1 apart (Section 2.1: a
 * composition is lowered to its primitives by bufferize rewrites): kind 10 is
 * the bias add alone, kind 11 the ReLU alone, each with microkernels of its
 * own, and kind 12 the Specs of kind 1 with one more rewrite per memory level:
 * a bufferize that splits the composition into the bias add writing an
 * intermediate in that level and the ReLU reading it.
 * Layouts (Section 2.4.2): besides row-major (0) and column-major (1), where a
 * lattice of kind 7 or 8 sets layout_coord to 2 a tensor may be packed in
 * strips of `strip` columns (2) and packed with odd-even shuffled strips (3);
 * orc_layout_offset writes the four buffer indexing expressions out.
 */
#define _GNU_SOURCE             /* qsort_r */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_INF   UINT64_MAX
#define ORC_NONE  0xFFFFu
#define ORC_LIMIT (((unsigned __int128)1) << 62)

enum { ORC_MAXL = 4, ORC_MAXOPS = 5, ORC_MAXD = 16, ORC_MAXMK = 8 };
enum { MK_SCALAR_FMA = 0, MK_BCAST_VEC_MULADD = 1, MK_BF16_DOT = 2,
       MK_SCALAR_ADDRELU = 3, MK_VEC_ADDRELU = 4,
       MK_SCALAR_MOVE = 5, MK_VECTOR_MOVE = 6, MK_VECTOR_MOVE_ALIGNED = 7,
       MK_SCALAR_ADD = 8, MK_VEC_ADD = 9, MK_SCALAR_RELU = 10, MK_VEC_RELU = 11 };
enum { KIND_M = 0, KIND_E = 1, KIND_F = 2, KIND_P = 3, KIND_B = 4, KIND_BE = 5, KIND_BF = 6,
       KIND_V = 7,    /* Move Specs */
       KIND_MV = 8,   /* a Matmul whose Moves are Move Specs of a kind 7 table */
       KIND_G = 9,    /* composition of two Matmuls (Section 2.1): (lhs x rhs1) x rhs2 accumulated into out */
       KIND_A = 10,   /* bias add: in (m x n), bias (n), out (m x n) */
       KIND_R = 11,   /* ReLU: in (m x n), out (m x n) */
       KIND_S = 12 }; /* bias add -> ReLU as kind 1, plus the bufferize between the two */
enum { ACC_READ = 0, ACC_RMW = 1, ACC_WRITE = 2 };

typedef struct {
  uint32_t n_levels;
  uint64_t capacity_bytes[ORC_MAXL];
  uint32_t load_coef[ORC_MAXL][ORC_MAXL][2];   /* [src][dst][same|transposed] */
  uint32_t store_coef[ORC_MAXL][ORC_MAXL][2];  /* [dst][src][same|transposed] */
  uint32_t convert_coef;
  uint32_t zero_coef[ORC_MAXL];
  uint32_t loop_overhead;
  uint32_t n_microkernels;
  uint32_t mk_kind[ORC_MAXMK];
  uint32_t mk_lanes[ORC_MAXMK];
  uint64_t mk_cost[ORC_MAXMK];
  uint32_t threads;                            /* hardware threads a parallel loop spreads over */
  uint32_t sync_cost;                          /* the constant s of a parallel loop */
  uint32_t level_weight[ORC_MAXL];             /* weight_level of m(t), Section 3 (kind 8) */
  uint32_t line_bytes;                         /* cache line: unit of lines(t) and of alignment (kinds 7, 8) */
  uint32_t strip;                              /* columns per strip of the packed layouts (kinds 7, 8; even) */
} orc_target;

typedef struct {
  uint32_t kind;
  uint32_t n_sizes[4];
  const uint32_t* sizes[4];                    /* b, m, k, n */
  uint8_t layout_coord[ORC_MAXOPS];            /* 0 none, 1 row-/column-major, 2 those and the two packed layouts */
  uint8_t dtype_coord[ORC_MAXOPS];
  uint8_t base_dtype_bytes[ORC_MAXOPS];
} orc_lattice;

/* A Spec (Section 2.2) reduced to the fields the lattices carry. */
typedef struct {
  uint32_t si[4];               /* index of b, m, k, n in the allowed-size lists */
  uint8_t level[ORC_MAXOPS];    /* per operand; kind F: level[4] = intermediate */
  uint8_t layout[ORC_MAXOPS];   /* 0 row-major, 1 column-major, 2 packed strips, 3 packed and shuffled strips */
  uint8_t bf16[ORC_MAXOPS];     /* 0 f32, 1 bf16 */
  uint8_t limit[ORC_MAXL];      /* kind B: per bounded level, index of the memory bound: 0 -> 0 bytes,
                                   q -> 2^(q-1) bytes */
  uint8_t contig[2];            /* kind V, per tensor (source, destination): number of inner physical
                                   dimensions whose values are adjacent in memory, 0..2, for a packed
                                   tensor (three physical dimensions) 0..3 (Section 2.4.3) */
  uint8_t aligned[2];           /* kind V: 1 = the tensor starts at a multiple of the cache line */
} spec_t;

typedef struct ctx {
  const orc_target* T;
  const orc_lattice* L;
  int kind, nops, nlv, ndim;
  uint32_t ext[ORC_MAXD];
  uint64_t stride[ORC_MAXD];
  int lay_axis[ORC_MAXOPS], dt_axis[ORC_MAXOPS];
  uint64_t n;
  uint64_t* cost;
  uint16_t* arg;
  uint8_t* done;
  uint32_t maxs, nmk, move_base, tile_base, buf_id, par_base;
  int parallel;                 /* kind P: a Matmul whose serial-only flag is off */
  int bounded;                  /* kinds 4..6: the Specs carry per-level memory bounds */
  int lim_axis[ORC_MAXL];       /* coordinate axis of level l's bound, -1 if the level is unbounded */
  int moves;                    /* kind 8: Moves are Move Specs, looked up in depM (a kind V table) */
  int split;                    /* kind 12: kind E plus bufferize(level); depM = the bias-add table, depE = the ReLU table */
  int packed;                   /* kinds 7, 8: some tensor has the four-layout coordinate (Move ids then hold 4 layout changes) */
  int abs_axis;                 /* kind V: first of the four axes contig(src), aligned(src), contig(dst), aligned(dst); -1 else */
  uint64_t n_rewrites, n_admissible;
  int overflow;
  const struct ctx* depM;
  const struct ctx* depE;
  uint32_t k_first;             /* kind F: where this lattice's k list starts within depM's */
} ctx;

/* ------------------------------------------------------------------ */
/* Coordinates (Section 4.1: Specs map to points of Z>=0^D).  Axis order:
 * size indices b,m,k,n; operand levels (kind F: then the intermediate's);
 * layout bits of the operands that have one; dtype bits likewise.  The dense
 * tables are in C order of that vector, last axis fastest. */
static int ctx_init(ctx* c, const orc_target* T, const orc_lattice* L) {
  memset(c, 0, sizeof *c);
  c->T = T; c->L = L; c->kind = (int)L->kind;
  if (c->kind < 0 || c->kind > KIND_S) return -1;
  c->abs_axis = -1;
  if (c->kind == KIND_MV) { c->kind = KIND_M; c->moves = 1; }     /* same operator, operands and coordinates as kind M */
  if (c->kind == KIND_S) { c->kind = KIND_E; c->split = 1; }      /* same operator, operands and coordinates as kind E */
  if (c->kind >= KIND_B && c->kind <= KIND_BF) { c->kind -= KIND_B; c->bounded = 1; }   /* kinds 4, 5, 6: M, E, F with memory bounds */
  if (c->kind == KIND_P) {      /* same operator, operands and coordinates as kind M */
    c->kind = KIND_M; c->parallel = 1;
    if (T->threads < 1) return -1;
  }
  if (T->n_levels < 1 || T->n_levels > ORC_MAXL) return -1;
  c->nops = c->kind == KIND_F || c->kind == KIND_G ? 4 : c->kind == KIND_V || c->kind == KIND_R ? 2 : 3;
  c->nlv = c->kind == KIND_F || c->kind == KIND_G ? 5 : c->kind == KIND_V || c->kind == KIND_R ? 2 : 3;
  if ((c->kind == KIND_V || c->moves) && T->line_bytes < 1) return -1;
  for (int i = 0; i < c->nops; i++) {
    if (L->layout_coord[i] > 2) return -1;
    if (L->layout_coord[i] == 2) {
      if (!(c->kind == KIND_V || c->moves) || T->strip < 2 || T->strip % 2) return -1;
      c->packed = 1;
    }
  }
  int d = 0;
  c->maxs = 0;
  for (int a = 0; a < 4; a++) {
    /* every list starts with 1, except the k list of a fused lattice: no rewrite of a fused Spec
     * changes k, so a fused lattice may cover any stretch of k values (a slab of the whole one) */
    if (L->n_sizes[a] < 1) return -1;
    if (L->sizes[a][0] != 1 && !(a == 2 && (L->kind == KIND_F || L->kind == KIND_BF))) return -1;
    for (uint32_t j = 1; j < L->n_sizes[a]; j++)
      if (L->sizes[a][j] <= L->sizes[a][j - 1]) return -1;
    c->ext[d++] = L->n_sizes[a];
    if (L->n_sizes[a] > c->maxs) c->maxs = L->n_sizes[a];
  }
  if (c->kind != KIND_M && c->kind != KIND_G && L->n_sizes[0] != 1) return -1;   /* no batch on E, F (kind G keeps p there) */
  if ((c->kind == KIND_E || c->kind == KIND_V || c->kind == KIND_A || c->kind == KIND_R) && L->n_sizes[2] != 1) return -1;   /* no k */
  if (c->moves && L->n_sizes[0] != 1) return -1;            /* operands of a kind 8 Matmul are two-dimensional */
  for (int i = 0; i < c->nlv; i++) c->ext[d++] = T->n_levels;
  /* Memory bounds (Section 2.2, field 5; Section 4.1: limits are powers of two): one axis per
   * level with a finite capacity; the values are 0, 1, 2, 4, ... up to the capacity. */
  for (int l = 0; l < ORC_MAXL; l++) c->lim_axis[l] = -1;
  if (c->bounded)
    for (uint32_t l = 0; l < T->n_levels; l++) {
      if (T->capacity_bytes[l] == UINT64_MAX) continue;
      uint32_t nq = 1;
      while (nq < 64 && ((uint64_t)1 << (nq - 1)) <= T->capacity_bytes[l]) nq++;
      if (nq > 255) return -1;
      c->lim_axis[l] = d; c->ext[d++] = nq;
    }
  if (c->kind == KIND_V) {      /* Section 2.4.3: the abstract values are part of a tensor specification */
    c->abs_axis = d;
    c->ext[d++] = c->packed ? 4 : 3; c->ext[d++] = 2; c->ext[d++] = c->packed ? 4 : 3; c->ext[d++] = 2;
  }
  for (int i = 0; i < ORC_MAXOPS; i++) { c->lay_axis[i] = -1; c->dt_axis[i] = -1; }
  for (int i = 0; i < c->nops; i++)
    if (L->layout_coord[i]) { c->lay_axis[i] = d; c->ext[d++] = L->layout_coord[i] == 2 ? 4 : 2; }
  for (int i = 0; i < c->nops; i++)
    if (L->dtype_coord[i]) {
      if (!(c->kind == KIND_V || (c->kind == KIND_M && i != 2))) return -1;   /* inputs of a Matmul, tensors of a Move */
      /* (kinds E, F, G: f32 throughout) */
      c->dt_axis[i] = d; c->ext[d++] = 2;
    }
  c->ndim = d;
  uint64_t s = 1;
  for (int a = d - 1; a >= 0; a--) { c->stride[a] = s; s *= c->ext[a]; }
  c->n = s;
  c->nmk = T->n_microkernels;
  c->move_base = c->nmk;
  c->tile_base = c->move_base + (uint32_t)c->nops * (T->n_levels - 1) * (c->packed ? 8 : 4);
  c->buf_id = c->tile_base + 4 * c->maxs;
  c->par_base = c->buf_id + 1;
  if ((c->parallel ? c->par_base + 4 * c->maxs : c->buf_id + T->n_levels) >= ORC_NONE) return -1;
  return 0;
}

static uint64_t spec_index(const ctx* c, const spec_t* s) {
  uint64_t x = 0;
  for (int a = 0; a < 4; a++) x += s->si[a] * c->stride[a];
  for (int i = 0; i < c->nlv; i++) x += s->level[i] * c->stride[4 + i];
  for (int i = 0; i < c->nops; i++) {
    if (c->lay_axis[i] >= 0) x += s->layout[i] * c->stride[c->lay_axis[i]];
    if (c->dt_axis[i] >= 0) x += s->bf16[i] * c->stride[c->dt_axis[i]];
  }
  for (int l = 0; l < ORC_MAXL; l++)
    if (c->lim_axis[l] >= 0) x += s->limit[l] * c->stride[c->lim_axis[l]];
  if (c->abs_axis >= 0)
    for (int t = 0; t < 2; t++)
      x += s->contig[t] * c->stride[c->abs_axis + 2 * t] + s->aligned[t] * c->stride[c->abs_axis + 2 * t + 1];
  return x;
}

static void spec_of_index(const ctx* c, uint64_t x, spec_t* s) {
  memset(s, 0, sizeof *s);
  uint32_t coord[ORC_MAXD];
  for (int a = 0; a < c->ndim; a++) { coord[a] = (uint32_t)(x / c->stride[a]); x %= c->stride[a]; }
  for (int a = 0; a < 4; a++) s->si[a] = coord[a];
  for (int i = 0; i < c->nlv; i++) s->level[i] = (uint8_t)coord[4 + i];
  for (int i = 0; i < c->nops; i++) {
    if (c->lay_axis[i] >= 0) s->layout[i] = (uint8_t)coord[c->lay_axis[i]];
    if (c->dt_axis[i] >= 0) s->bf16[i] = (uint8_t)coord[c->dt_axis[i]];
    else s->bf16[i] = c->L->base_dtype_bytes[i] == 2;
  }
  for (int l = 0; l < ORC_MAXL; l++)
    if (c->lim_axis[l] >= 0) s->limit[l] = (uint8_t)coord[c->lim_axis[l]];
  if (c->abs_axis >= 0)
    for (int t = 0; t < 2; t++) {
      s->contig[t] = (uint8_t)coord[c->abs_axis + 2 * t];
      s->aligned[t] = (uint8_t)coord[c->abs_axis + 2 * t + 1];
    }
}

/* ------------------------------------------------------------------ */
/* Shapes.  Section 2: dimensions are batch, m, k, n; lhs is b x m x k, rhs is
 * b x k x n, the output b x m x n.  Kind E: in (m x n), bias (n), out (m x n).
 * Kind F: lhs, rhs, bias, out, and the intermediate (m x n, f32). */
static void dims_of(const ctx* c, const spec_t* s, uint64_t d[4]) {
  for (int a = 0; a < 4; a++) d[a] = c->L->sizes[a][s->si[a]];
}

static uint64_t numel(const ctx* c, const spec_t* s, int op) {
  uint64_t d[4]; dims_of(c, s, d);
  uint64_t b = d[0], m = d[1], k = d[2], n = d[3];
  switch (c->kind) {
    case KIND_M: return op == 0 ? b * m * k : op == 1 ? b * k * n : b * m * n;
    case KIND_E:
    case KIND_A: return op == 1 ? n : m * n;
    case KIND_R: return m * n;
    case KIND_V: return m * n;                                                    /* source and destination: rows x cols */
    case KIND_G: /* b holds p, the dimension the two Matmuls share: lhs m x k, rhs1 k x p, rhs2 p x n, out m x n, mid m x p */
      return op == 0 ? m * k : op == 1 ? k * b : op == 2 ? b * n : op == 3 ? m * n : m * b;
    default:     return op == 0 ? m * k : op == 1 ? k * n : op == 2 ? n : m * n; /* 3 = out, 4 = mid */
  }
}

static int access_of(const ctx* c, int op) {
  if (c->kind == KIND_M) return op == 2 ? ACC_RMW : ACC_READ;     /* accumulating output */
  if (c->kind == KIND_G) return op == 3 ? ACC_RMW : ACC_READ;     /* the second Matmul accumulates into out */
  return op == c->nops - 1 ? ACC_WRITE : ACC_READ;
}

/* ------------------------------------------------------------------ */
/* Layouts (Section 2.4.2): a layout maps the coordinates (i, j) of a rows x cols tensor to a
 * buffer offset, a bijection onto 0 .. rows*cols-1.  Row-major and column-major nest the two
 * logical dimensions; the packed layout adds a strip dimension of s columns: strips one after
 * the other, inside a strip the rows, inside a row of a strip its s columns; the shuffled one
 * permutes the columns of a strip by the odd-even shuffle sigma(s, x) = 2 (x mod s/2) + floor(2x / s).
 * (The printed strip formula multiplies floor(j / s) by the row count alone; a strip holds
 * rows * s values, so that term is rows * s * floor(j / s) here: only then is the map a bijection.) */
uint64_t orc_layout_offset(uint32_t layout, uint64_t rows, uint64_t cols, uint64_t s, uint64_t i, uint64_t j) {
  switch (layout) {
    case 0: return cols * i + j;
    case 1: return rows * j + i;
    case 2: return rows * s * (j / s) + s * i + j % s;
    default: { uint64_t x = j % s; return rows * s * (j / s) + s * i + 2 * (x % (s / 2)) + 2 * x / s; }
  }
}

/* Physical dimensions of a rows x cols tensor, outermost first; returns how many there are.  A
 * packed tensor consists of whole strips, or (a tile cut out of one strip) of the same part of
 * every row of one strip. */
static int phys_dims(uint32_t layout, uint64_t rows, uint64_t cols, uint64_t s, uint64_t d[3]) {
  if (layout == 0) { d[0] = rows; d[1] = cols; return 2; }
  if (layout == 1) { d[0] = cols; d[1] = rows; return 2; }
  if (cols >= s) { d[0] = cols / s; d[1] = rows; d[2] = s; }
  else { d[0] = 1; d[1] = rows; d[2] = cols; }
  return 3;
}

static int layout_fits(const ctx* c, uint32_t layout, uint64_t cols) {
  uint64_t s = c->T->strip;
  return layout < 2 || cols % s == 0 || (cols < s && s % cols == 0);
}

/* The most inner physical dimensions whose values can be adjacent.  The rows of a part of a strip
 * lie a whole strip apart, and in a shuffled strip the columns of such a part are not adjacent
 * either. */
static int max_contig(uint32_t layout, uint64_t cols, uint64_t s) {
  if (layout < 2) return 2;
  if (cols >= s) return 3;
  if (layout == 2) return 1;
  return cols == 1 ? 1 : 0;
}

/* rows and columns of operand i of a kind 8 Matmul: lhs m x k, rhs k x n, out m x n */
static void operand_rows_cols(const uint64_t d4[4], int i, uint64_t* rows, uint64_t* cols) {
  *rows = i == 1 ? d4[2] : d4[1];
  *cols = i == 0 ? d4[2] : d4[3];
}

/* A Spec is admissible when the tensors resident in each level fit that level
 * (the per-level memory bound of Section 2.2, applied to the Spec's own
 * operands; kind F also counts its intermediate). */
static int admissible(const ctx* c, const spec_t* s) {
  if (c->bounded) return 1;     /* the bounds, not the operands' footprint, limit what a Spec may do */
  if (c->packed) {              /* no such tensor: a packed layout with a broken strip, more adjacent dimensions than there are */
    uint64_t d4[4], rows, cols; dims_of(c, s, d4);
    for (int i = 0; i < c->nops; i++) {
      if (c->kind == KIND_V) { rows = d4[1]; cols = d4[3]; } else operand_rows_cols(d4, i, &rows, &cols);
      if (!layout_fits(c, s->layout[i], cols)) return 0;
      if (c->kind == KIND_V && s->contig[i] > max_contig(s->layout[i], cols, c->T->strip)) return 0;
      if (c->kind != KIND_V && s->layout[i] >= 2 && cols % c->T->strip) return 0;    /* a whole (fresh) tensor: whole strips */
    }
  }
  if (c->kind == KIND_V) return 1;   /* both tensors of a Move exist already: whoever placed them answered for their size */
  for (uint32_t l = 0; l < c->T->n_levels; l++) {
    unsigned __int128 bytes = 0;
    for (int i = 0; i < c->nops; i++)
      if (s->level[i] == l) bytes += (unsigned __int128)numel(c, s, i) * (s->bf16[i] ? 2 : 4);
    if ((c->kind == KIND_F || c->kind == KIND_G) && s->level[4] == l) bytes += (unsigned __int128)numel(c, s, 4) * 4;
    if (c->T->capacity_bytes[l] != UINT64_MAX && bytes > c->T->capacity_bytes[l]) return 0;
  }
  return 1;
}

/* a * sub + b with INF absorbing and the 2^62 range check. */
static uint64_t affine(ctx* c, uint64_t a, uint64_t sub, unsigned __int128 b) {
  if (sub == ORC_INF) return ORC_INF;
  unsigned __int128 v = (unsigned __int128)a * sub + b;
  if (v >= ORC_LIMIT) { c->overflow = 1; return ORC_INF; }
  return (uint64_t)v;
}

/* Microkernel applicability and repetition count (Section 2, Microkernel
 * Selection; Figure 1: BroadcastVecMultAdd on an RF, VRF, VRF 1x1x1x16 Spec).
 * Returns 0 when the predicate fails, else the number of repetitions. */
static uint64_t mk_reps(const ctx* c, const spec_t* s, int j) {
  uint64_t d[4]; dims_of(c, s, d);
  uint64_t b = d[0], m = d[1], k = d[2], n = d[3];
  uint32_t lanes = c->T->mk_lanes[j];
  const uint8_t* lv = s->level; const uint8_t* ly = s->layout; const uint8_t* bf = s->bf16;
  switch (c->T->mk_kind[j]) {
    case MK_SCALAR_FMA:
      if (c->kind != KIND_M) return 0;
      if (b != 1 || m != 1 || k != 1 || n != 1) return 0;
      if (lv[0] != 0 || lv[1] != 0 || lv[2] != 0) return 0;
      if (bf[0] || bf[1] || bf[2]) return 0;
      return 1;
    case MK_BCAST_VEC_MULADD:
      if (c->kind != KIND_M) return 0;
      if (b != 1 || m != 1 || k != 1 || n % lanes != 0) return 0;
      if (lv[0] != 0 || lv[1] != 1 || lv[2] != 1) return 0;
      if (bf[0] || bf[1] || bf[2]) return 0;
      /* rhs, out row-major; one row in whole packed strips is the same sequence of values */
      for (int i = 1; i <= 2; i++)
        if (!(ly[i] == 0 || (ly[i] == 2 && c->T->strip % lanes == 0))) return 0;
      return n / lanes;
    case MK_BF16_DOT:
      if (c->kind != KIND_M) return 0;
      if (b != 1 || m != 1 || n != 1 || k % lanes != 0) return 0;
      if (lv[0] != 1 || lv[1] != 1 || lv[2] != 0) return 0;
      if (!bf[0] || !bf[1] || bf[2]) return 0;
      if (c->lay_axis[1] >= 0 && ly[1] != 1) return 0;  /* rhs column-major */
      return k / lanes;
    case MK_SCALAR_ADDRELU:
      if (c->kind != KIND_E) return 0;
      if (m != 1 || n != 1) return 0;
      if (lv[0] != 0 || lv[1] != 0 || lv[2] != 0) return 0;
      return 1;
    case MK_VEC_ADDRELU:
      if (c->kind != KIND_E) return 0;
      if (m != 1 || n % lanes != 0) return 0;
      if (lv[0] != 1 || lv[1] != 1 || lv[2] != 1) return 0;
      if (ly[0] != 0 || ly[2] != 0) return 0;
      return n / lanes;
    /* The two halves of the bias-add + ReLU, for the lattices of kinds 10 and 11. */
    case MK_SCALAR_ADD:
      if (c->kind != KIND_A) return 0;
      if (m != 1 || n != 1) return 0;
      if (lv[0] != 0 || lv[1] != 0 || lv[2] != 0) return 0;
      return 1;
    case MK_VEC_ADD:
      if (c->kind != KIND_A) return 0;
      if (m != 1 || n % lanes != 0) return 0;
      if (lv[0] != 1 || lv[1] != 1 || lv[2] != 1) return 0;
      if (ly[0] != 0 || ly[2] != 0) return 0;
      return n / lanes;
    case MK_SCALAR_RELU:
      if (c->kind != KIND_R) return 0;
      if (m != 1 || n != 1) return 0;
      if (lv[0] != 0 || lv[1] != 0) return 0;
      return 1;
    case MK_VEC_RELU:
      if (c->kind != KIND_R) return 0;
      if (m != 1 || n % lanes != 0) return 0;
      if (lv[0] != 1 || lv[1] != 1) return 0;
      if (ly[0] != 0 || ly[1] != 0) return 0;
      return n / lanes;
    /* Move microkernels (Section 2: select(VectorMove), a vector load or store).  m = rows,
     * n = columns of the moved tensor; operand 0 is the source, 1 the destination. */
    case MK_SCALAR_MOVE:                 /* one element, between any two places; converts if the types differ */
      if (c->kind != KIND_V) return 0;
      if (m != 1 || n != 1) return 0;
      if (!bf[0] && bf[1]) return 0;     /* no narrowing */
      return 1;
    case MK_VECTOR_MOVE:
    case MK_VECTOR_MOVE_ALIGNED:         /* one row of whole vectors between the vector registers (level 1) and a slower level */
      if (c->kind != KIND_V) return 0;
      if (m != 1 || n % lanes != 0) return 0;
      if (!((lv[0] == 1 && lv[1] > 1) || (lv[1] == 1 && lv[0] > 1))) return 0;
      /* the row's values are the inner dimension: row-major, or strips of whole vectors; shuffled
       * strips only to shuffled strips (the vectors then hold the same values on both sides) */
      for (int t = 0; t < 2; t++)
        if (!(ly[t] == 0 || (ly[t] >= 2 && (n < c->T->strip || c->T->strip % lanes == 0)))) return 0;
      if ((ly[0] == 3) != (ly[1] == 3)) return 0;
      if (bf[0] != bf[1]) return 0;                         /* no conversion */
      if (s->contig[0] < 1 || s->contig[1] < 1) return 0;   /* ... and adjacent in memory */
      if (c->T->mk_kind[j] == MK_VECTOR_MOVE_ALIGNED && !(s->aligned[0] && s->aligned[1])) return 0;
      return n / lanes;
    default: return 0;
  }
}

/* Section 2.4.3, for a tile of r2 x c2 cut out of tensor t (0 source, 1 destination) of a Move
 * Spec of r x c: contiguousness counts the inner physical dimensions whose values are adjacent;
 * cutting the inner dimension leaves only the inner one adjacent.  A tile is known to be aligned
 * only if the tensor was aligned and contiguous and every suffix of the tile's physical
 * dimensions is a whole number of cache lines. */
static void tile_tensor(const ctx* c, const spec_t* s, int t, uint64_t r, uint64_t col, uint64_t r2, uint64_t c2,
                        uint8_t* contig, uint8_t* aligned) {
  uint64_t e = s->bf16[t] ? 2 : 4, line = c->T->line_bytes, strip = c->T->strip ? c->T->strip : 1;
  uint64_t whole[3], part[3];
  int nd = phys_dims(s->layout[t], r, col, strip, whole);
  phys_dims(s->layout[t], r2, c2, strip, part);
  /* the tile's values over its inner j dimensions are adjacent while the j-1 innermost are uncut */
  int uncut = 0;
  while (uncut < nd && part[nd - 1 - uncut] == whole[nd - 1 - uncut]) uncut++;
  int keep = 1 + uncut, most = max_contig(s->layout[t], c2, strip);
  if (keep > most) keep = most;
  *contig = (uint8_t)(s->contig[t] < keep ? s->contig[t] : keep);
  int lines_ok = s->layout[t] < 2 || c2 >= strip;        /* a part of a strip is not known to be aligned */
  uint64_t suffix = e;
  for (int q = nd - 1; q >= 0; q--) { suffix *= part[q]; if (suffix % line) lines_ok = 0; }
  *aligned = s->aligned[t] && s->contig[t] == nd && lines_ok;
}

/* Section 3: m(t) = lines(t) * weight of t's level * (2 if t is not contiguous, else 1), for a
 * tensor of `elems` elements of `bytes` bytes that is contiguous and aligned (the operands of the
 * Matmul lattices carry no contiguousness or alignment coordinate: they are taken as fresh). */
static unsigned __int128 m_of(const ctx* c, uint64_t elems, uint32_t bytes, uint32_t level) {
  unsigned __int128 b = (unsigned __int128)elems * bytes;
  unsigned __int128 lines = (b + c->T->line_bytes - 1) / c->T->line_bytes;
  return lines * c->T->level_weight[level];
}

static uint64_t solve(ctx* c, const spec_t* s);

static void consider(ctx* c, uint64_t cand, uint32_t id, uint64_t* best, uint16_t* arg) {
  c->n_rewrites++;
  if (cand < *best) { *best = cand; *arg = (uint16_t)id; }   /* first strict minimum */
}

/* Section 4: evaluate every applicable rewrite of one Spec, in id order. */
static void expand(ctx* c, const spec_t* s, uint64_t* best_out, uint16_t* arg_out) {
  const orc_target* T = c->T;
  uint64_t best = ORC_INF; uint16_t arg = ORC_NONE;
  uint32_t NL = T->n_levels;

  /* A. select(microkernel): a leaf costing k_p per repetition. */
  for (uint32_t j = 0; j < c->nmk; j++) {
    uint64_t reps = mk_reps(c, s, (int)j);
    if (!reps) continue;
    consider(c, affine(c, 0, 0, (unsigned __int128)T->mk_cost[j] * reps), j, &best, &arg);
  }

  /* B. move an operand to a strictly faster level (alloc-binding: the move's
   * own cost plus the cost of the body Spec).  A Move Spec has no such rewrite. */
  for (int i = 0; i < (c->kind == KIND_V ? 0 : c->nops); i++) {
    int acc = access_of(c, i);
    uint32_t src = s->level[i];
    for (uint32_t dst = 0; dst + 1 < NL; dst++)
      for (int x = 0; x < (c->packed ? 4 : 2); x++)        /* the Move leaves the operand in layout (its own) xor x */
        for (int cv = 0; cv < 2; cv++) {
          if (dst >= src) continue;
          if (x && c->lay_axis[i] < 0) continue;
          if (x >= 2 && c->L->layout_coord[i] != 2) continue;
          if (cv && !(c->dt_axis[i] >= 0 && s->bf16[i] && acc == ACC_READ)) continue;
          spec_t sub = *s;
          sub.level[i] = (uint8_t)dst;
          sub.layout[i] ^= (uint8_t)x;
          if (cv) sub.bf16[i] = 0;
          uint32_t id = c->move_base + (((uint32_t)i * (NL - 1) + dst) * (c->packed ? 4 : 2) + (uint32_t)x) * 2 + (uint32_t)cv;
          if (c->moves) {
            /* Section 2, Memory Movement: the alloc-binding holds a load Move Spec (unless the
             * operand is only written), the body, and a store Move Spec (if it is written);
             * Section 3: it costs m(src) + m(dest) plus its children. */
            uint64_t d4[4]; dims_of(c, s, d4);
            uint64_t rows, cols, pd[3];
            operand_rows_cols(d4, i, &rows, &cols);
            spec_t mv; memset(&mv, 0, sizeof mv);
            mv.si[1] = i == 1 ? s->si[2] : s->si[1];
            mv.si[3] = i == 0 ? s->si[2] : s->si[3];
            /* both tensors fresh: every physical dimension adjacent, aligned (Section 2.4.3) */
            uint8_t top_own = (uint8_t)phys_dims(s->layout[i], rows, cols, T->strip ? T->strip : 1, pd);
            uint8_t top_new = (uint8_t)phys_dims(sub.layout[i], rows, cols, T->strip ? T->strip : 1, pd);
            mv.aligned[0] = mv.aligned[1] = 1;
            uint64_t c_load = 0, c_store = 0;
            if (acc != ACC_WRITE) {
              mv.level[0] = (uint8_t)src; mv.level[1] = (uint8_t)dst;
              mv.layout[0] = s->layout[i]; mv.layout[1] = sub.layout[i];
              mv.contig[0] = top_own; mv.contig[1] = top_new;
              mv.bf16[0] = s->bf16[i]; mv.bf16[1] = sub.bf16[i];
              c_load = c->depM->cost[spec_index(c->depM, &mv)];
            }
            if (acc != ACC_READ) {
              mv.level[0] = (uint8_t)dst; mv.level[1] = (uint8_t)src;
              mv.layout[0] = sub.layout[i]; mv.layout[1] = s->layout[i];
              mv.contig[0] = top_new; mv.contig[1] = top_own;
              mv.bf16[0] = sub.bf16[i]; mv.bf16[1] = s->bf16[i];
              c_store = c->depM->cost[spec_index(c->depM, &mv)];
            }
            unsigned __int128 fixed = m_of(c, rows * cols, s->bf16[i] ? 2 : 4, src) + m_of(c, rows * cols, sub.bf16[i] ? 2 : 4, dst);
            uint64_t cand = ORC_INF;
            if (c_load != ORC_INF && c_store != ORC_INF) cand = affine(c, 1, solve(c, &sub), fixed + c_load + c_store);
            consider(c, cand, id, &best, &arg);
            continue;
          }
          uint64_t coef = 0;
          if (acc != ACC_WRITE) { if (!T->load_coef[src][dst][x]) continue; coef += T->load_coef[src][dst][x]; }
          if (acc != ACC_READ) { if (!T->store_coef[dst][src][x]) continue; coef += T->store_coef[dst][src][x]; }
          if (cv) coef += T->convert_coef;
          if (c->bounded && c->lim_axis[dst] >= 0) {
            /* Section 2.4.4: the Move allocates the operand's buffer in dst; the body may use
             * what is left of dst's bound, snapped down to a power of two (or zero). */
            unsigned __int128 bytes = (unsigned __int128)numel(c, s, i) * (sub.bf16[i] ? 2 : 4);
            uint64_t have = s->limit[dst] ? (uint64_t)1 << (s->limit[dst] - 1) : 0;
            if (bytes > have) continue;
            uint64_t left = have - (uint64_t)bytes;
            uint8_t q = 0;
            while (q < 64 && ((uint64_t)1 << q) <= left) q++;      /* left = 0 -> 0; else floor(log2) + 1 */
            sub.limit[dst] = q;
          }
          uint64_t cand = affine(c, 1, solve(c, &sub), (unsigned __int128)coef * numel(c, s, i));
          consider(c, cand, id, &best, &arg);
        }
  }

  /* C. tile one dimension to a smaller allowed size dividing it: a loop of
   * trips iterations around the smaller Spec, plus the loop constant s. */
  for (int d = 0; d < 4; d++) {
    if (c->kind != KIND_M && (d == 0 || d == 2)) continue;   /* E, F: only m and n */
    uint32_t cur = c->L->sizes[d][s->si[d]];
    for (uint32_t j = 0; j < s->si[d]; j++) {
      uint32_t t = c->L->sizes[d][j];
      if (cur % t) continue;
      spec_t sub = *s;
      sub.si[d] = j;
      if (c->kind == KIND_V) {
        uint64_t d4[4]; dims_of(c, s, d4);
        uint64_t r2 = d == 1 ? t : d4[1], c2 = d == 3 ? t : d4[3];
        for (int ts = 0; ts < 2; ts++) tile_tensor(c, s, ts, d4[1], d4[3], r2, c2, &sub.contig[ts], &sub.aligned[ts]);
      }
      uint64_t cand = affine(c, cur / t, solve(c, &sub), T->loop_overhead);
      consider(c, cand, c->tile_base + (uint32_t)d * c->maxs + j, &best, &arg);
    }
  }

  /* D. bufferize (kind F): a pipeline of the Matmul writing the intermediate
   * and the bias-add+ReLU reading it; cost = sum of the children plus
   * initialising the accumulated intermediate. */
  if (c->kind == KIND_F) {
    spec_t ms; memset(&ms, 0, sizeof ms);
    spec_t es; memset(&es, 0, sizeof es);
    for (int a = 0; a < 4; a++) ms.si[a] = s->si[a];
    ms.si[2] += c->k_first;
    ms.level[0] = s->level[0]; ms.level[1] = s->level[1]; ms.level[2] = s->level[4];
    ms.layout[0] = s->layout[0]; ms.layout[1] = s->layout[1]; ms.layout[2] = 0;
    es.si[1] = s->si[1]; es.si[3] = s->si[3];
    es.level[0] = s->level[4]; es.level[1] = s->level[2]; es.level[2] = s->level[3];
    es.layout[0] = 0; es.layout[2] = s->layout[3];
    int fits = 1;
    if (c->bounded) {
      /* Section 2.4.4: the pipeline allocates the intermediate in its level; both stages may use
       * what is left of that level's bound, snapped down to a power of two (or zero). */
      memcpy(ms.limit, s->limit, sizeof ms.limit);
      memcpy(es.limit, s->limit, sizeof es.limit);
      uint32_t lm = s->level[4];
      if (c->lim_axis[lm] >= 0) {
        unsigned __int128 bytes = (unsigned __int128)numel(c, s, 4) * 4;
        uint64_t have = s->limit[lm] ? (uint64_t)1 << (s->limit[lm] - 1) : 0;
        if (bytes > have) fits = 0;
        else {
          uint64_t left = have - (uint64_t)bytes;
          uint8_t q = 0;
          while (q < 64 && ((uint64_t)1 << q) <= left) q++;
          ms.limit[lm] = es.limit[lm] = q;
        }
      }
    }
    if (fits) {
      uint64_t cm = c->depM->cost[spec_index(c->depM, &ms)];
      uint64_t ce = c->depE->cost[spec_index(c->depE, &es)];
      uint64_t cand = ORC_INF;
      if (cm != ORC_INF && ce != ORC_INF) {
        unsigned __int128 v = (unsigned __int128)T->zero_coef[s->level[4]] * numel(c, s, 4) + cm + ce;
        if (v >= ORC_LIMIT) c->overflow = 1; else cand = (uint64_t)v;
      }
      consider(c, cand, c->buf_id, &best, &arg);
    }
  }

  /* D'. bufferize of two composed Matmuls (kind G, Section 2.1): the first Matmul writes the
   * intermediate (m x p, f32, row-major, initialised first), the second accumulates its product
   * with rhs2 into out.  Both are Specs of the Matmul table: (m, k, p) and (m, p, n). */
  if (c->kind == KIND_G) {
    spec_t m1; memset(&m1, 0, sizeof m1);
    spec_t m2; memset(&m2, 0, sizeof m2);
    m1.si[1] = s->si[1]; m1.si[2] = s->si[2]; m1.si[3] = s->si[0];            /* m, k, n := p */
    m1.level[0] = s->level[0]; m1.level[1] = s->level[1]; m1.level[2] = s->level[4];
    m1.layout[0] = s->layout[0]; m1.layout[1] = s->layout[1];
    m2.si[1] = s->si[1]; m2.si[2] = s->si[0]; m2.si[3] = s->si[3];            /* m, k := p, n */
    m2.level[0] = s->level[4]; m2.level[1] = s->level[2]; m2.level[2] = s->level[3];
    m2.layout[1] = s->layout[2]; m2.layout[2] = s->layout[3];
    uint64_t c1 = c->depM->cost[spec_index(c->depM, &m1)];
    uint64_t c2 = c->depM->cost[spec_index(c->depM, &m2)];
    uint64_t cand = ORC_INF;
    if (c1 != ORC_INF && c2 != ORC_INF) {
      unsigned __int128 v = (unsigned __int128)T->zero_coef[s->level[4]] * numel(c, s, 4) + c1 + c2;
      if (v >= ORC_LIMIT) c->overflow = 1; else cand = (uint64_t)v;
    }
    consider(c, cand, c->buf_id, &best, &arg);
  }

  /* D''. bufferize of the bias-add + ReLU (kind 12, Section 2.1), one rewrite per level l of the
   * intermediate (m x n, f32, row-major): the bias add writes it, the ReLU reads it; a pipeline
   * costs the sum of its stages (Section 3; nothing accumulates into this intermediate, so it is
   * not initialised).  The intermediate must fit level l next to the Spec's operands there. */
  if (c->split) {
    for (uint32_t l = 0; l < NL; l++) {
      unsigned __int128 bytes = (unsigned __int128)numel(c, s, 0) * 4;      /* the intermediate: as large as in */
      for (int i = 0; i < 3; i++) if (s->level[i] == l) bytes += (unsigned __int128)numel(c, s, i) * 4;
      if (T->capacity_bytes[l] != UINT64_MAX && bytes > T->capacity_bytes[l]) continue;
      spec_t as; memset(&as, 0, sizeof as);
      spec_t rs; memset(&rs, 0, sizeof rs);
      as.si[1] = rs.si[1] = s->si[1]; as.si[3] = rs.si[3] = s->si[3];
      as.level[0] = s->level[0]; as.level[1] = s->level[1]; as.level[2] = (uint8_t)l;
      as.layout[0] = s->layout[0];
      rs.level[0] = (uint8_t)l; rs.level[1] = s->level[2];
      rs.layout[1] = s->layout[2];
      uint64_t ca = c->depM->cost[spec_index(c->depM, &as)];
      uint64_t cr = c->depE->cost[spec_index(c->depE, &rs)];
      uint64_t cand = ORC_INF;
      if (ca != ORC_INF && cr != ORC_INF) {
        unsigned __int128 v = (unsigned __int128)ca + cr;
        if (v >= ORC_LIMIT) c->overflow = 1; else cand = (uint64_t)v;
      }
      consider(c, cand, c->buf_id + l, &best, &arg);
    }
  }

  /* E. parallel loop (kind P, Section 3: ceil(trips / threads) * c(body) + s).
   * The body is the serial-only Spec of the smaller shape (Section 2.2: the
   * flag limits an implementation to one hardware thread), so its cost comes
   * from the serial table.  Not over k: its iterations accumulate into the
   * same output elements. */
  if (c->parallel) {
    for (int d = 0; d < 4; d++) {
      if (d == 2) continue;
      uint32_t cur = c->L->sizes[d][s->si[d]];
      for (uint32_t j = 0; j < s->si[d]; j++) {
        uint32_t t = c->L->sizes[d][j];
        if (cur % t) continue;
        spec_t sub = *s;
        sub.si[d] = j;
        uint64_t trips = cur / t, rounds = (trips + T->threads - 1) / T->threads;
        uint64_t body = c->depM->cost[spec_index(c->depM, &sub)];
        consider(c, affine(c, rounds, body, T->sync_cost), c->par_base + (uint32_t)d * c->maxs + j, &best, &arg);
      }
    }
  }
  *best_out = best; *arg_out = arg;
}

static uint64_t solve(ctx* c, const spec_t* s) {
  uint64_t x = spec_index(c, s);
  if (c->done[x]) return c->cost[x];
  uint64_t best = ORC_INF; uint16_t arg = ORC_NONE;
  if (admissible(c, s)) { c->n_admissible++; expand(c, s, &best, &arg); }
  c->cost[x] = best; c->arg[x] = arg; c->done[x] = 1;
  return best;
}

static int same_sizes(const orc_lattice* a, int da, const orc_lattice* b, int db) {
  if (a->n_sizes[da] != b->n_sizes[db]) return 0;
  return memcmp(a->sizes[da], b->sizes[db], a->n_sizes[da] * sizeof(uint32_t)) == 0;
}

/* Fill the whole table.  `goals` (optional) are linear indices solved first,
 * in the given order; every remaining point is then solved in index order.
 * Returns 0, -1 (bad arguments) or -6 (a finite cost reached 2^62). */
int orc_solve(const orc_target* T, const orc_lattice* L,
              const orc_lattice* LM, const uint64_t* costM,
              const orc_lattice* LE, const uint64_t* costE,
              const uint64_t* goals, uint64_t n_goals,
              uint64_t* cost, uint16_t* arg,
              uint64_t* n_admissible, uint64_t* n_rewrites) {
  ctx c, cm, ce;
  if (ctx_init(&c, T, L)) return -1;
  if (c.kind == KIND_F) {
    if (!LM || !LE || !costM || !costE) return -1;
    if (ctx_init(&cm, T, LM) || ctx_init(&ce, T, LE)) return -1;
    if (cm.kind != KIND_M || cm.parallel || ce.kind != KIND_E) return -1;
    if (cm.bounded != c.bounded || ce.bounded != c.bounded) return -1;      /* bounds on all three tables or on none */
    /* a tensor whose layout the fused lattice distinguishes must have that coordinate in the table it is looked up in */
    if ((c.lay_axis[0] >= 0 && cm.lay_axis[0] < 0) || (c.lay_axis[1] >= 0 && cm.lay_axis[1] < 0) ||
        (c.lay_axis[3] >= 0 && ce.lay_axis[2] < 0)) return -1;
    if (!same_sizes(L, 1, LM, 1) || !same_sizes(L, 3, LM, 3)) return -1;
    {
      /* the k list: a stretch of consecutive entries of the Matmul table's */
      uint32_t o = 0;
      while (o < LM->n_sizes[2] && LM->sizes[2][o] != L->sizes[2][0]) o++;
      if (o + L->n_sizes[2] > LM->n_sizes[2]) return -1;
      if (memcmp(LM->sizes[2] + o, L->sizes[2], L->n_sizes[2] * sizeof(uint32_t))) return -1;
      c.k_first = o;
    }
    if (LM->n_sizes[0] != 1) return -1;
    if (!same_sizes(L, 1, LE, 1) || !same_sizes(L, 3, LE, 3)) return -1;
    for (int i = 0; i < 3; i++) if (cm.dt_axis[i] >= 0 || LM->base_dtype_bytes[i] != 4) return -1;
    cm.cost = (uint64_t*)costM; ce.cost = (uint64_t*)costE;
    c.depM = &cm; c.depE = &ce;
  }
  if (c.split) {                /* the two stages: the bias-add table and the ReLU table */
    if (!LM || !LE || !costM || !costE) return -1;
    if (ctx_init(&cm, T, LM) || ctx_init(&ce, T, LE)) return -1;
    if (cm.kind != KIND_A || ce.kind != KIND_R) return -1;
    if (!same_sizes(L, 1, LM, 1) || !same_sizes(L, 3, LM, 3) || !same_sizes(L, 1, LE, 1) || !same_sizes(L, 3, LE, 3)) return -1;
    if ((c.lay_axis[0] >= 0 && cm.lay_axis[0] < 0) || (c.lay_axis[2] >= 0 && ce.lay_axis[1] < 0)) return -1;
    cm.cost = (uint64_t*)costM; ce.cost = (uint64_t*)costE;
    c.depM = &cm; c.depE = &ce;
  }
  if (c.kind == KIND_G) {       /* both stages are Specs of one Matmul table */
    if (!LM || !costM) return -1;
    if (ctx_init(&cm, T, LM)) return -1;
    if (cm.kind != KIND_M || cm.parallel || cm.bounded || cm.moves || LM->n_sizes[0] != 1) return -1;
    /* m from m; the lists of k, p and n, and the table's k and n lists, must all be the same */
    if (!same_sizes(L, 1, LM, 1) || !same_sizes(L, 2, LM, 2) || !same_sizes(L, 0, LM, 2) || !same_sizes(L, 0, LM, 3) ||
        !same_sizes(L, 3, LM, 3)) return -1;
    if ((c.lay_axis[0] >= 0 && cm.lay_axis[0] < 0) || (c.lay_axis[1] >= 0 && cm.lay_axis[1] < 0) ||
        (c.lay_axis[2] >= 0 && cm.lay_axis[1] < 0) || (c.lay_axis[3] >= 0 && cm.lay_axis[2] < 0)) return -1;
    for (int i = 0; i < 3; i++) if (cm.dt_axis[i] >= 0 || LM->base_dtype_bytes[i] != 4) return -1;
    cm.cost = (uint64_t*)costM;
    c.depM = &cm;
  }
  if (c.moves) {                /* the Move Specs: a kind V table over the same sizes */
    if (!LM || !costM) return -1;
    if (ctx_init(&cm, T, LM)) return -1;
    if (cm.kind != KIND_V) return -1;
    /* every operand's shape must be in the Move lattice: rows from m and k, columns from k and n */
    if (!same_sizes(L, 1, LM, 1) || !same_sizes(L, 2, LM, 1) || !same_sizes(L, 2, LM, 3) || !same_sizes(L, 3, LM, 3)) return -1;
    int any_lay = 0, any_dt = 0;
    for (int i = 0; i < 3; i++) { any_lay |= c.lay_axis[i] >= 0; any_dt |= c.dt_axis[i] >= 0 || L->base_dtype_bytes[i] == 2; }
    if (any_lay && (cm.lay_axis[0] < 0 || cm.lay_axis[1] < 0)) return -1;
    if (c.packed && (LM->layout_coord[0] != 2 || LM->layout_coord[1] != 2)) return -1;
    if (any_dt && (cm.dt_axis[0] < 0 || cm.dt_axis[1] < 0)) return -1;
    if (cm.dt_axis[0] < 0 && (LM->base_dtype_bytes[0] != 4 || LM->base_dtype_bytes[1] != 4)) return -1;
    cm.cost = (uint64_t*)costM;
    c.depM = &cm;
  }
  if (c.parallel) {             /* the serial-only Specs: the kind M table of the same lattice */
    if (!LM || !costM) return -1;
    if (ctx_init(&cm, T, LM)) return -1;
    if (cm.kind != KIND_M || cm.parallel || cm.ndim != c.ndim) return -1;
    for (int d = 0; d < 4; d++) if (!same_sizes(L, d, LM, d)) return -1;
    for (int i = 0; i < 3; i++)
      if (cm.lay_axis[i] != c.lay_axis[i] || cm.dt_axis[i] != c.dt_axis[i] ||
          LM->base_dtype_bytes[i] != L->base_dtype_bytes[i]) return -1;
    cm.cost = (uint64_t*)costM;
    c.depM = &cm;
  }
  c.cost = cost; c.arg = arg;
  c.done = (uint8_t*)calloc(c.n, 1);
  if (!c.done) return -2;
  spec_t s;
  for (uint64_t g = 0; g < n_goals; g++) {
    if (goals[g] >= c.n) { free(c.done); return -1; }
    spec_of_index(&c, goals[g], &s); solve(&c, &s);
  }
  for (uint64_t x = 0; x < c.n; x++) { spec_of_index(&c, x, &s); solve(&c, &s); }
  free(c.done);
  if (n_admissible) *n_admissible = c.n_admissible;
  if (n_rewrites) *n_rewrites = c.n_rewrites;
  return c.overflow ? -6 : 0;
}

/* Geometry of the table: number of axes, extents, and the merge order used by
 * orc_merge (the memory-bound axes, then n, k, m, b, the level axes,
 * layout bits and dtype bits, each group last to first). */
int orc_geometry(const orc_target* T, const orc_lattice* L, uint32_t* ndim,
                 uint32_t* ext, uint32_t* merge_order, uint32_t* ids) {
  ctx c;
  if (ctx_init(&c, T, L)) return -1;
  *ndim = (uint32_t)c.ndim;
  for (int a = 0; a < c.ndim; a++) ext[a] = c.ext[a];
  int nlay = 0, nlim = 0;
  for (int i = 0; i < c.nops; i++) nlay += c.lay_axis[i] >= 0;
  for (int l = 0; l < ORC_MAXL; l++) nlim += c.lim_axis[l] >= 0;
  if (c.abs_axis >= 0) nlim = 4;   /* a Move lattice's abstract-value axes stand where the memory bounds do */
  int q = 0, first = 4 + c.nlv;
  for (int a = first + nlim - 1; a >= first; a--) merge_order[q++] = (uint32_t)a;                /* memory bounds */
  for (int a = 3; a >= 0; a--) merge_order[q++] = (uint32_t)a;                                   /* n, k, m, b */
  for (int a = first - 1; a >= 4; a--) merge_order[q++] = (uint32_t)a;                           /* levels */
  first += nlim;
  for (int a = first + nlay - 1; a >= first; a--) merge_order[q++] = (uint32_t)a;                /* layout bits */
  for (int a = c.ndim - 1; a >= first + nlay; a--) merge_order[q++] = (uint32_t)a;               /* dtype bits */
  if (ids) { ids[0] = c.move_base; ids[1] = c.tile_base; ids[2] = c.buf_id; ids[3] = c.maxs; }
  return 0;
}

/* ------------------------------------------------------------------ */
/* Values that the two box lists compare (Section 4.1): the decision itself,
 * and the cost normalised to the Spec's volume b*m*k*n, kept as an exact
 * reduced fraction v0/v1.  INF is (2^64-1, 0). */
static uint64_t gcd64(uint64_t a, uint64_t b) { while (b) { uint64_t t = a % b; a = b; b = t; } return a; }

int orc_cost_values(const orc_target* T, const orc_lattice* L, const uint64_t* cost,
                    uint64_t* v0, uint64_t* v1) {
  ctx c;
  if (ctx_init(&c, T, L)) return -1;
  spec_t s; uint64_t d[4];
  for (uint64_t x = 0; x < c.n; x++) {
    if (cost[x] == ORC_INF) { v0[x] = ORC_INF; v1[x] = 0; continue; }
    spec_of_index(&c, x, &s); dims_of(&c, &s, d);
    uint64_t vol = d[0] * d[1] * d[2] * d[3];
    uint64_t g = gcd64(cost[x], vol);
    v0[x] = cost[x] / g; v1[x] = vol / g;
  }
  return 0;
}

typedef struct { uint16_t lo[ORC_MAXD], hi[ORC_MAXD]; uint64_t v0, v1; } orc_box;

/* What a comparison needs besides the two boxes (handed to qsort_r, so that the merge keeps no
 * state between calls). */
typedef struct { int axis, ndim; } sort_key;

/* Group key: value, then lo/hi on every axis but the merge axis; inside a
 * group order by lo on the merge axis. */
static int cmp_group(const void* pa, const void* pb, void* pk) {
  const orc_box* a = (const orc_box*)pa; const orc_box* b = (const orc_box*)pb;
  const sort_key* k = (const sort_key*)pk;
  if (a->v0 != b->v0) return a->v0 < b->v0 ? -1 : 1;
  if (a->v1 != b->v1) return a->v1 < b->v1 ? -1 : 1;
  for (int j = 0; j < k->ndim; j++) {
    if (j == k->axis) continue;
    if (a->lo[j] != b->lo[j]) return a->lo[j] < b->lo[j] ? -1 : 1;
    if (a->hi[j] != b->hi[j]) return a->hi[j] < b->hi[j] ? -1 : 1;
  }
  if (a->lo[k->axis] != b->lo[k->axis]) return a->lo[k->axis] < b->lo[k->axis] ? -1 : 1;
  return 0;
}

static int same_group(const orc_box* a, const orc_box* b, const sort_key* k) {
  if (a->v0 != b->v0 || a->v1 != b->v1) return 0;
  for (int j = 0; j < k->ndim; j++) {
    if (j == k->axis) continue;
    if (a->lo[j] != b->lo[j] || a->hi[j] != b->hi[j]) return 0;
  }
  return 1;
}

static int cmp_lo(const void* pa, const void* pb, void* pk) {
  const orc_box* a = (const orc_box*)pa; const orc_box* b = (const orc_box*)pb;
  const sort_key* k = (const sort_key*)pk;
  for (int j = 0; j < k->ndim; j++)
    if (a->lo[j] != b->lo[j]) return a->lo[j] < b->lo[j] ? -1 : 1;
  return 0;
}

/* One merge pass along `axis`: join every maximal chain of boxes of one group
 * in which each box starts right after the previous one ends. */
static uint64_t merge_axis(orc_box* b, uint64_t n, int axis, int ndim) {
  if (n == 0) return 0;
  sort_key key = {axis, ndim};
  qsort_r(b, n, sizeof *b, cmp_group, &key);
  uint64_t w = 0;
  for (uint64_t r = 1; r < n; r++) {
    if (same_group(&b[w], &b[r], &key) && b[r].lo[axis] == b[w].hi[axis] + 1) b[w].hi[axis] = b[r].hi[axis];
    else b[++w] = b[r];
  }
  return w + 1;
}

/* Canonical box decomposition of a dense table of values (v0[x], v1[x]).
 * Starts from one unit box per cell and applies merge_axis for each axis of
 * merge_order in turn; the result is sorted by lo (first axis most
 * significant).  With first_pass_by_lines != 0 the first axis is merged by
 * walking each line of cells along it, which forms the same chains as the
 * group-and-sort pass does on unit boxes but needs one box per run, not per
 * cell (the two are compared in the tests).  Returns a malloc'ed array. */
int64_t orc_merge(uint32_t ndim, const uint32_t* ext, const uint32_t* merge_order, uint32_t n_merge,
                  const uint64_t* v0, const uint64_t* v1, int first_pass_by_lines, orc_box** out) {
  uint64_t stride[ORC_MAXD], n = 1;
  for (int a = (int)ndim - 1; a >= 0; a--) { stride[a] = n; n *= ext[a]; }
  orc_box* b; uint64_t nb = 0; uint32_t first = 0;
  if (first_pass_by_lines && n_merge > 0) {
    uint32_t ax = merge_order[0];
    uint64_t cap = 1024;
    b = (orc_box*)malloc(cap * sizeof *b);
    if (!b) return -2;
    for (uint64_t x = 0; x < n; x++) {
      uint32_t ca = (uint32_t)((x / stride[ax]) % ext[ax]);
      if (ca > 0 && v0[x - stride[ax]] == v0[x] && v1[x - stride[ax]] == v1[x]) continue;  /* not a run start */
      uint32_t e = ca;
      while (e + 1 < ext[ax] && v0[x + (e + 1 - ca) * stride[ax]] == v0[x] && v1[x + (e + 1 - ca) * stride[ax]] == v1[x]) e++;
      if (nb == cap) { cap *= 2; b = (orc_box*)realloc(b, cap * sizeof *b); if (!b) return -2; }
      memset(&b[nb], 0, sizeof *b);
      uint64_t r = x;
      for (uint32_t a = 0; a < ndim; a++) { b[nb].lo[a] = b[nb].hi[a] = (uint16_t)(r / stride[a]); r %= stride[a]; }
      b[nb].hi[ax] = (uint16_t)e; b[nb].v0 = v0[x]; b[nb].v1 = v1[x];
      nb++;
    }
    first = 1;
  } else {
    b = (orc_box*)malloc((n ? n : 1) * sizeof *b);
    if (!b) return -2;
    for (uint64_t x = 0; x < n; x++) {
      memset(&b[x], 0, sizeof *b);
      uint64_t r = x;
      for (uint32_t a = 0; a < ndim; a++) { b[x].lo[a] = b[x].hi[a] = (uint16_t)(r / stride[a]); r %= stride[a]; }
      b[x].v0 = v0[x]; b[x].v1 = v1[x];
    }
    nb = n;
  }
  for (uint32_t q = first; q < n_merge; q++) nb = merge_axis(b, nb, (int)merge_order[q], (int)ndim);
  sort_key by_lo = {-1, (int)ndim};
  qsort_r(b, nb, sizeof *b, cmp_lo, &by_lo);
  *out = b;
  return (int64_t)nb;
}

void orc_free(void* p) { free(p); }

/* Paint the boxes back into dense arrays; cover[x] counts how many boxes
 * contain cell x (1 everywhere for a valid decomposition). */
int orc_decompress(uint32_t ndim, const uint32_t* ext, const orc_box* b, uint64_t nb,
                   uint64_t* v0, uint64_t* v1, uint8_t* cover) {
  uint64_t stride[ORC_MAXD], n = 1;
  for (int a = (int)ndim - 1; a >= 0; a--) { stride[a] = n; n *= ext[a]; }
  memset(cover, 0, n);
  for (uint64_t i = 0; i < nb; i++) {
    uint32_t c[ORC_MAXD];
    for (uint32_t a = 0; a < ndim; a++) {
      if (b[i].lo[a] > b[i].hi[a] || b[i].hi[a] >= ext[a]) return -1;
      c[a] = b[i].lo[a];
    }
    for (;;) {
      uint64_t x = 0;
      for (uint32_t a = 0; a < ndim; a++) x += c[a] * stride[a];
      v0[x] = b[i].v0; v1[x] = b[i].v1;
      if (cover[x] < 255) cover[x]++;
      int a = (int)ndim - 1;
      while (a >= 0) { if (c[a] < b[i].hi[a]) { c[a]++; break; } c[a] = b[i].lo[a]; a--; }
      if (a < 0) break;
    }
  }
  return 0;
}
