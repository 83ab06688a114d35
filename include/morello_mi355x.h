/*
 * morello_mi355x.h -- C ABI of the MI355X (gfx950) memo-table solver.
 *
 * The library fills, bottom-up on the GPU, the memoization table of the
 * dynamic-programming synthesis of Section 4 of the paper over a lattice of
 * Matmul Specs, and compresses it into boxes as in Section 4.1.
 *
 * Conventions
 *   - Every function returns an int32_t status: MRL_OK or a negative MRL_E_*.
 *     No exception or abort crosses the boundary.  mrl_last_error() returns a
 *     thread-local, library-owned string describing the last failure.
 *   - Handles (mrl_target, mrl_table) are created by the library and
 *     destroyed by the caller.  Descriptor structs are copied: the library
 *     keeps no caller host pointer after a call returns.
 *   - "host" / "device" is stated for every pointer.  Device buffers handed to
 *     mrl_solve stay owned by the caller and must outlive the mrl_table.
 *   - All costs are unsigned 64-bit integers; MRL_INF marks a Spec with no
 *     implementation; finite costs are kept below 2^62.
 */
#ifndef MORELLO_MI355X_H
#define MORELLO_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MRL_OK = 0,
  MRL_E_INVAL = -1,     /* malformed descriptor or argument                    */
  MRL_E_NOMEM = -2,     /* scratch buffer too small / host allocation failed   */
  MRL_E_HIP = -3,       /* a HIP runtime call failed                           */
  MRL_E_RANGE = -4,     /* coordinate outside the lattice                      */
  MRL_E_BUFSZ = -5,     /* caller's output buffer too small; *n_out = needed   */
  MRL_E_OVERFLOW = -6   /* a finite cost reached 2^62                          */
};

#define MRL_INF  UINT64_MAX     /* cost of a Spec without implementation */
#define MRL_NONE 0xFFFFu        /* its rewrite id                        */

enum { MRL_MAX_LEVELS = 4, MRL_MAX_OPERANDS = 5, MRL_MAX_DIMS = 16, MRL_MAX_MK = 8,
       MRL_MAX_SIZES = 255 };

/* ---------------------------------------------------------------------------
 * Target (Section 2.2: memory levels ordered RF, VRF, L1, GL with per-level
 * bounds; Section 3: microkernel costs k_p, loop constant s, per-level Move
 * weights).  Level 0 is the fastest.  A Move goes to a strictly lower level
 * index only, and costs coef * (elements of the operand): load_coef for an
 * operand that is read, store_coef for one that is written, both for the
 * accumulated output of a MatmulAccum (their sum must fit 32 bits, or creating
 * a lattice fails with MRL_E_INVAL).  A zero coefficient forbids the Move.
 */
typedef enum {
  MRL_MK_SCALAR_FMA = 0,        /* 1x1x1x1 MatmulAccum, all operands in level 0, f32          */
  MRL_MK_BCAST_VEC_MULADD = 1,  /* Figure 1: b=m=k=1, n % lanes == 0, lhs level 0, rhs and
                                   out level 1, f32, row-major                               */
  MRL_MK_BF16_DOT = 2,          /* m=n=1, k % lanes == 0, bf16 lhs/rhs in level 1 (rhs
                                   column-major), f32 out in level 0                         */
  MRL_MK_SCALAR_ADDRELU = 3,    /* bias-add+ReLU, m=n=1, all in level 0                        */
  MRL_MK_VEC_ADDRELU = 4,       /* bias-add+ReLU, m=1, n % lanes == 0, all level 1, row-major  */
  /* Move Specs (Section 2: select(VectorMove)); m = rows, n = columns of the moved tensor */
  MRL_MK_SCALAR_MOVE = 5,       /* 1x1, between any two places, any layouts; converts bf16 to f32
                                   when the types differ (never the other way)                  */
  MRL_MK_VECTOR_MOVE = 6,       /* one row, n % lanes == 0, between level 1 and a level above 1
                                   (either way), both row-major, same type, the inner dimension
                                   of both tensors adjacent in memory (contiguousness >= 1)     */
  MRL_MK_VECTOR_MOVE_ALIGNED = 7, /* the same, and both tensors aligned                          */
  /* the two halves of the bias-add + ReLU, for BIAS_ADD and RELU lattices */
  MRL_MK_SCALAR_ADD = 8,        /* bias add, m=n=1, all in level 0                             */
  MRL_MK_VEC_ADD = 9,           /* bias add, m=1, n % lanes == 0, all level 1, in and out row-major */
  MRL_MK_SCALAR_RELU = 10,      /* ReLU, m=n=1, both in level 0                                */
  MRL_MK_VEC_RELU = 11          /* ReLU, m=1, n % lanes == 0, both level 1, row-major          */
} mrl_mk_kind;

typedef struct { uint32_t kind; uint32_t lanes; uint64_t cost; } mrl_microkernel;

typedef struct {
  uint32_t n_levels;                                          /* 1..4                              */
  uint64_t capacity_bytes[MRL_MAX_LEVELS];                    /* UINT64_MAX = unbounded            */
  uint32_t load_coef[MRL_MAX_LEVELS][MRL_MAX_LEVELS][2];      /* [src][dst][same|transposed], dst<src */
  uint32_t store_coef[MRL_MAX_LEVELS][MRL_MAX_LEVELS][2];     /* [dst][src][same|transposed]       */
  uint32_t convert_coef;                                      /* bf16->f32, per element, added to a Move */
  uint32_t zero_coef[MRL_MAX_LEVELS];                         /* per element of the bufferized intermediate */
  uint32_t loop_overhead;                                     /* s of Section 3, paid by every loop */
  uint32_t n_microkernels;
  mrl_microkernel mk[MRL_MAX_MK];                             /* order = rewrite-id order          */
  uint32_t threads;                                           /* Section 3: hardware threads a parallel
                                                                 loop spreads its trips over; >= 1 for a
                                                                 MATMUL_PARALLEL lattice, else ignored */
  uint32_t sync_cost;                                         /* Section 3: constant of a parallel loop */
  uint32_t level_weight[MRL_MAX_LEVELS];                      /* Section 3: weight of a level in m(t), the cost
                                                                 of an alloc-binding (MATMUL_MOVES)            */
  uint32_t line_bytes;                                        /* cache line: unit of lines(t) in m(t) and of
                                                                 alignment; >= 1 for MOVE and MATMUL_MOVES     */
  uint32_t strip;                                             /* Section 2.4.2: columns per strip of the packed
                                                                 layouts; even and >= 2 where a lattice has
                                                                 layout_coord 2, else ignored                  */
} mrl_target_desc;

typedef struct mrl_target mrl_target;

/* desc: host.  *out receives a new handle.  MRL_E_INVAL on a malformed descriptor. */
int32_t mrl_target_create(const mrl_target_desc* desc, mrl_target** out);
void mrl_target_destroy(mrl_target* t);

/* ---------------------------------------------------------------------------
 * Lattice of Specs (Section 2.2 reduced to integer coordinates, Section 4.1).
 * Coordinate vector x, in this order:
 *   index of b, m, k, n in the allowed-size lists;
 *   memory level of each operand (FUSED, MATMUL_CHAIN: then the intermediate's level);
 *   (the BOUNDED kinds: one memory-bound index per level of finite capacity;)
 *   one layout coordinate per operand with layout_coord: 0 row-major, 1
 *   column-major, and where layout_coord is 2 (MOVE, MATMUL_MOVES) also 2
 *   packed in strips and 3 packed with shuffled strips (see PACKED LAYOUTS);
 *   one dtype bit (0 f32, 1 bf16) per operand with dtype_coord.
 * Dense tables are in C order of x (last coordinate fastest).
 *
 * Operands.  MATMUL_ACCUM: lhs (b*m*k, read), rhs (b*k*n, read), out (b*m*n,
 * accumulated).  BIAS_ADD_RELU: in (m*n, read), bias (n, read), out (m*n,
 * written); b and k must be pinned to 1.  FUSED_MM_ADD_RELU (Section 2.1,
 * Matmul -> bias add -> ReLU split once by bufferize): lhs, rhs, bias (read),
 * out (written), intermediate m*n f32; b pinned to 1; only m and n are tiled.
 * Its k list need not start with 1: no rewrite of a fused Spec changes k, so the
 * lattice may cover any stretch of consecutive entries of its MATMUL_ACCUM
 * dep's k list (a slab; the slabs of a lattice too large for one table can be
 * solved one after the other into the same buffers).
 * Where the FUSED lattice has a layout coordinate (lhs, rhs, out), the dep in
 * which that tensor is looked up must have one too (MRL_E_INVAL else).
 * MATMUL_PARALLEL (Section 2.2: the serial-only flag; Section 3: the loop
 * rule with threads): the MATMUL_ACCUM Specs with the flag off.  Same
 * operands, coordinates and rewrites as MATMUL_ACCUM, plus a parallel loop
 * over b, m or n (not k, whose iterations accumulate into the same output):
 * ceil(trips / threads) * cost of the body + sync_cost, where the body is
 * the serial-only Spec of the smaller shape.  The serial-only Specs are the
 * MATMUL_ACCUM table of the same lattice, passed as the one dependency: the
 * flag is kept as two tables rather than as an axis of one.
 * MATMUL_BOUNDED (Section 2.2, field 5; Section 2.4.4; Section 4.1: limits are
 * powers of two): the MATMUL_ACCUM Specs with a peak-memory bound per level
 * of finite capacity as further coordinates, placed after the operand levels
 * and before the layout bits, one axis per such level in level order.
 * Coordinate q stands for a bound of 0 bytes (q = 0) or 2^(q-1) bytes, up to
 * the largest power of two within the capacity.  There is no admissibility
 * test by footprint; instead a Move needs the moved operand's bytes (at the
 * dtype it has after the Move) within the destination level's bound, and its
 * body Spec gets what is left, rounded down to a power of two (or zero).
 * Tiles keep the bounds.  Rewrite ids as for MATMUL_ACCUM; no deps.
 * BIAS_ADD_RELU_BOUNDED and FUSED_BOUNDED: the same for the other two
 * operators.  A bufferize allocates the intermediate (4*m*n bytes) in its
 * level: it needs that much of the level's bound, and both stages get the
 * rest, rounded down (Section 2.4.4, pipelines).  FUSED_BOUNDED takes deps =
 * {MATMUL_BOUNDED table, BIAS_ADD_RELU_BOUNDED table}.
 * MOVE (Section 2.2: a Move Spec copies a tensor into another that may differ
 * in memory level, layout and data type; it is implemented like any Spec, by
 * loops over smaller Move Specs and move microkernels).  Two tensors, source
 * (operand 0) and destination (operand 1), of m x n elements (rows, columns;
 * b and k pinned to 1).  Coordinates: the two size indices; the two levels;
 * then, where the BOUNDED kinds have their bounds, four axes with the abstract
 * values of Section 2.4.3: contiguousness of the source (0..2: how many inner
 * physical dimensions have their values adjacent in memory), aligned flag of
 * the source, and the same for the destination; layout and dtype bits of both
 * tensors.  Rewrites: the move microkernels and tiles of m and n.  A tile of
 * r2 x c2 keeps a tensor's contiguousness unless its inner dimension (columns
 * if row-major, rows else) is cut, which leaves at most 1; it is aligned only
 * if the tensor was aligned and contiguous (2) and the tile's inner extent in
 * bytes is a multiple of line_bytes.  No admissibility test (both tensors
 * exist already); no deps.
 * MATMUL_MOVES (Section 2, Memory Movement; Section 3): the MATMUL_ACCUM Specs
 * (b pinned to 1), except that moving an operand does not cost a coefficient
 * per element: the alloc-binding costs m(src) + m(dest) plus its children,
 * which are a load Move Spec (unless the operand is only written), the body,
 * and a store Move Spec (if it is written).  m(t) = cache lines of t *
 * level_weight[level of t]; the operands count as contiguous and aligned
 * (these lattices have no such coordinates), so lines = ceil(bytes /
 * line_bytes).  The Move Specs' costs come from the one dep, a MOVE table of
 * the same target whose m and n size lists both equal this lattice's m, k and
 * n lists (which must be equal), with layout bits on both tensors if any
 * operand here has one and dtype bits on both if any operand here has one or
 * is bf16.  load_coef / store_coef / convert_coef are not used.
 * MATMUL_CHAIN (Section 2.1: a Spec may be a composition of sub-Specs, split
 * by bufferize into a pipeline around an intermediate tensor; Section 3: a
 * pipeline costs the sum of its stages): (lhs x rhs1) x rhs2 accumulated into
 * out.  sizes[0] holds p, the dimension the two Matmuls share, so x starts
 * with the indices of p, m, k, n.  Operands: lhs (m*k, read), rhs1 (k*p,
 * read), rhs2 (p*n, read), out (m*n, accumulated); then the level of the
 * intermediate (m*p, f32, row-major), as for FUSED.  Rewrites: Moves of the
 * four operands, tiles of m and n, and one bufferize (same id as FUSED's):
 * zero_coef[level of the intermediate] * m*p + the MATMUL_ACCUM Spec (1, m,
 * k, p) with out := the intermediate + the MATMUL_ACCUM Spec (1, m, p, n)
 * with lhs := the intermediate.  A Spec is admissible when its operands and
 * the intermediate fit their levels.  deps = {MATMUL_ACCUM table}, f32, b
 * pinned to 1, whose m list equals this lattice's and whose k and n lists
 * both equal this lattice's p, k and n lists (which must be equal); where an
 * operand here has a layout coordinate, the position it takes in the dep
 * (lhs, rhs1 -> lhs, rhs; rhs2, out -> rhs, out) must have one too.
 * PACKED LAYOUTS (Section 2.4.2; MOVE and MATMUL_MOVES lattices, layout_coord
 * 2 on a tensor).  Element (i, j) of a rows x cols tensor lies at offset
 * cols*i + j (0, row-major), rows*j + i (1, column-major), rows*s*floor(j/s) +
 * s*i + (j mod s) (2, packed in strips of s = target.strip columns) or the same
 * with sigma(s, j mod s) = 2*((j mod s) mod s/2) + floor(2*(j mod s)/s) in place
 * of (j mod s) (3, strips odd-even shuffled).  A packed tensor has three
 * physical dimensions (strips, rows, columns of a strip), so in a MOVE lattice
 * with a packed tensor the contiguousness axes have 4 values (0..3).  A packed
 * tensor consists of whole strips (cols a multiple of s); a tile of it may also
 * be the same part of every row of one strip (cols a divisor of s), of which at
 * most the part itself is adjacent (contiguousness <= 1; 0 in a shuffled strip
 * unless the part is one column) and which is never known to be aligned.  A
 * Spec with a tensor that does not exist in this sense has no implementation
 * and does not count as admissible.  A tile keeps min(contiguousness, 1 + the
 * number of innermost physical dimensions it takes whole, the limit above); it
 * is aligned if the tensor was aligned and contiguous in all its dimensions,
 * every suffix product of the tile's physical dimensions times the element size
 * is a multiple of line_bytes, and it is no part of a strip.  Vector moves take
 * rows of row-major tensors and of packed ones (whole strips: s a multiple of
 * the lanes), shuffled strips only when both tensors are shuffled;
 * MRL_MK_BCAST_VEC_MULADD takes rhs and out row-major or packed (not
 * shuffled) in strips that are a multiple of its lanes.  In a MATMUL_MOVES
 * lattice an operand with layout_coord 2 may be moved into any of the four
 * layouts (operands are whole tensors: a packed one needs cols a multiple of
 * s), its MOVE dep then needs layout_coord 2 on both tensors, and Move ids
 * are ((operand*(n_levels-1) + dst)*4 + (old layout xor new layout))*2 +
 * convert for every operand of the lattice.
 * BIAS_ADD, RELU, BIAS_ADD_RELU_SPLIT (Section 2.1: compositions are lowered
 * to their primitives by bufferize rewrites; here the second split of the
 * Matmul -> bias add -> ReLU pipeline, between the add and the ReLU).
 * BIAS_ADD: the operands and coordinates of BIAS_ADD_RELU (in m*n, bias n,
 * out m*n written); the microkernels that apply are MRL_MK_SCALAR_ADD and
 * MRL_MK_VEC_ADD.  RELU: in (m*n, read), out (m*n, written); b and k pinned
 * to 1; microkernels MRL_MK_SCALAR_RELU and MRL_MK_VEC_RELU.
 * BIAS_ADD_RELU_SPLIT: the BIAS_ADD_RELU Specs with the same rewrites and
 * ids, plus, for every memory level l in which an intermediate (m*n, f32,
 * row-major) fits next to those of the Spec's operands that live in l, a
 * bufferize with id (FUSED's bufferize id) + l: the BIAS_ADD Spec (in, bias,
 * intermediate at l) + the RELU Spec (intermediate at l, out); nothing
 * accumulates into this intermediate, so it is not initialised.  deps =
 * {BIAS_ADD table, RELU table} with this lattice's m and n lists, a layout
 * coordinate on in (BIAS_ADD) / out (RELU) where this lattice has one.  A
 * FUSED lattice takes a BIAS_ADD_RELU_SPLIT table as its second dep like a
 * BIAS_ADD_RELU table: its programs then hold both splits.
 */
typedef enum { MRL_KIND_MATMUL_ACCUM = 0, MRL_KIND_BIAS_ADD_RELU = 1,
               MRL_KIND_FUSED_MM_ADD_RELU = 2, MRL_KIND_MATMUL_PARALLEL = 3,
               MRL_KIND_MATMUL_BOUNDED = 4, MRL_KIND_BIAS_ADD_RELU_BOUNDED = 5,
               MRL_KIND_FUSED_BOUNDED = 6, MRL_KIND_MOVE = 7, MRL_KIND_MATMUL_MOVES = 8,
               MRL_KIND_MATMUL_CHAIN = 9, MRL_KIND_BIAS_ADD = 10, MRL_KIND_RELU = 11,
               MRL_KIND_BIAS_ADD_RELU_SPLIT = 12 } mrl_kind;

typedef struct {
  uint32_t kind;
  uint32_t n_sizes[4];                        /* 1..MRL_MAX_SIZES each                        */
  const uint32_t* sizes[4];                   /* host; ascending, sizes[d][0] == 1 (but see FUSED) */
  uint8_t layout_coord[MRL_MAX_OPERANDS];     /* 0 none, 1 row-/column-major, 2 also the packed layouts
                                                 (2 bits); layout and dtype bits together: at most 4
                                                 (6 for the MOVE, MATMUL_MOVES and BOUNDED kinds)   */
  uint8_t dtype_coord[MRL_MAX_OPERANDS];      /* inputs of a Matmul, both tensors of a MOVE   */
  uint8_t base_dtype_bytes[MRL_MAX_OPERANDS]; /* 4 or 2; used when the operand has no dtype bit */
} mrl_lattice_desc;

/* Number of coordinates and their extents (host outputs; extents has room for MRL_MAX_DIMS). */
int32_t mrl_geometry(const mrl_target* t, const mrl_lattice_desc* lat,
                     uint32_t* n_dims, uint32_t* extents, uint64_t* n_specs);

/* ---------------------------------------------------------------------------
 * Solve = fill (Section 4, bottom-up over dependency levels) + compress
 * (Section 4.1).  For every Spec the table holds
 *   cost   = min over applicable rewrites of (affine rewrite cost of Section 3
 *            applied to the costs of the rewrite's sub-Specs),
 *   argmin = the lowest rewrite id reaching that minimum (see mrl_rewrite_decode),
 * or (MRL_INF, MRL_NONE) when the Spec's operands do not fit their levels or
 * no complete program exists.
 */
typedef struct {
  uint64_t n_specs, n_admissible, n_rewrites; /* rewrites enumerated over all admissible Specs */
  uint32_t n_levels_run;                      /* dependency levels = fill launches             */
  float fill_ms, compress_ms;                 /* device time, HIP events on the given stream   */
  uint64_t n_decision_boxes, n_cost_boxes;
  uint64_t scratch_used;                      /* bytes of d_scratch actually needed            */
  float prefill_ms;                           /* the part of fill_ms before the first dependency
                                                 level: work lists and the (MRL_INF, MRL_NONE)
                                                 written over the whole table; 0 for BOUNDED kinds */
} mrl_stats;

/* Sizes of the device buffers mrl_solve needs.  scratch_bytes is sufficient for
 * any table contents; mrl_solve accepts less and fails with MRL_E_NOMEM if the
 * data turn out to need more. */
int32_t mrl_table_bytes(const mrl_target* t, const mrl_lattice_desc* lat,
                        size_t* cost_bytes, size_t* argmin_bytes, size_t* scratch_bytes);

typedef struct mrl_table mrl_table;

/* deps: host array of solved tables a FUSED lattice reads: {MATMUL_ACCUM table,
 * BIAS_ADD_RELU table} with the same m, k, n (m, n) size lists and target;
 * MATMUL_PARALLEL: {MATMUL_ACCUM table}; MATMUL_MOVES: {MOVE table};
 * MATMUL_CHAIN: {MATMUL_ACCUM table}; BIAS_ADD_RELU_SPLIT: {BIAS_ADD table,
 * RELU table}; NULL / 0 otherwise.  d_cost (uint64 per Spec), d_argmin (uint16 per Spec) and
 * d_scratch are DEVICE pointers, 256-byte aligned, owned by the caller and
 * referenced by *out until mrl_table_destroy.  hip_stream: a hipStream_t (or
 * NULL for the default stream); part of the work runs on a helper stream of
 * the library (default priority) that is ordered after and before the given
 * one, and the call returns after both have drained.  Calls from different
 * host threads (on different streams) may overlap, e.g. for lattices that do
 * not depend on each other; calls for the same (target, lattice) take turns.
 * stats: host, optional. */
int32_t mrl_solve(const mrl_target* t, const mrl_lattice_desc* lat,
                  const mrl_table* const* deps, uint32_t n_deps,
                  void* d_cost, void* d_argmin, void* d_scratch, size_t scratch_bytes,
                  void* hip_stream, mrl_table** out, mrl_stats* stats);
void mrl_table_destroy(mrl_table* tab);

/* Several lattices in one call (Section 4: the search of a Spec needs the memo
 * table entries of its sub-Specs, here the dense tables of the lattices it reads,
 * not their compressed form of Section 4.1).  Job j is what mrl_solve would do
 * with the same arguments, its deps given as indices of EARLIER jobs.  Every job
 * runs from a host thread of its own on its own stream (all different; default
 * priority); a job starts as soon as the FILL of its deps is queued: its work
 * lists and its pre-fill, which read no other table, run beside those fills, and
 * its dependency levels are ordered behind them on the device by an event (such a
 * job's fill_ms leaves out the time between the two in which it only waited); a
 * dep is compressed once the jobs that read it
 * have queued their own fill: its compression overlaps with their work instead of
 * holding it up, and independent jobs overlap as with mrl_solve from several
 * threads.  The last job runs on the calling thread.  No two jobs may be the
 * same lattice (MRL_E_INVAL).  jobs, out (n_jobs handles) and stats (n_jobs entries,
 * optional) are host arrays.  On success every out[j] is a table as from
 * mrl_solve.  On failure the status and message are those of the first job that
 * failed ("job <j>: ..."), no table is left and every out[j] is NULL.  The call
 * returns after all jobs have ended and their streams have drained. */
enum { MRL_MAX_JOBS = 16 };
typedef struct {
  const mrl_lattice_desc* lattice;
  uint32_t n_deps;
  uint32_t deps[2];                           /* indices of earlier jobs, in mrl_solve's dep order */
  void* d_cost;                               /* device, as for mrl_solve                           */
  void* d_argmin;
  void* d_scratch;
  size_t scratch_bytes;
  void* hip_stream;                           /* a hipStream_t; no two jobs share one               */
} mrl_job;
int32_t mrl_solve_graph(const mrl_target* t, const mrl_job* jobs, uint32_t n_jobs,
                        mrl_table** out, mrl_stats* stats);

/* ---------------------------------------------------------------------------
 * Query (Section 4: a Spec that the memo table already holds is answered from
 * it).  specs, cost_out, rewrite_out: host arrays of n.  Calls on one table from
 * several host threads take turns (they stage through the table's scratch buffer
 * and stream); so do those of mrl_schedule, which asks through this call. */
typedef struct { uint32_t x[MRL_MAX_DIMS]; } mrl_coord;
int32_t mrl_query(const mrl_table* tab, const mrl_coord* specs, size_t n,
                  uint64_t* cost_out, uint16_t* rewrite_out);

/* mrl_query for callers that cannot allocate: tight serving loops, harnesses
 * that forbid hipMalloc (and host allocation) once they are set up.  Same
 * arguments, answers and errors as mrl_query, but nothing is allocated, on the
 * device or on the host: the indices and answers are staged through an array of
 * MRL_NOALLOC_MAX_QUERIES * 18 bytes that the library holds in device memory of
 * every GPU it runs on, from load until the process ends, instead of through the
 * table's scratch buffer.  n must be at most MRL_NOALLOC_MAX_QUERIES
 * (MRL_E_INVAL else).  Every call on a GPU uses that GPU's one array and
 * overwrites what the call before left there; calls from several host threads of
 * one process take turns for it inside the library (work of another origin that
 * used the array while a call runs would race with it).  The table's device
 * buffers must be on the current device. */
enum { MRL_NOALLOC_MAX_QUERIES = 4096 };
int32_t mrl_query_noalloc(const mrl_table* tab, const mrl_coord* specs, size_t n,
                          uint64_t* cost_out, uint16_t* rewrite_out);

/* Rewrite ids, ascending = tie-break priority:
 *   [0, n_mk)                       select(microkernel j)
 *   then ((operand*(n_levels-1) + dst)*2 + transposed)*2 + convert   Moves (with packed layouts: *4 + the
 *                                                                    layout change, see PACKED LAYOUTS;
 *                                                                    mrl_rewrite.transposed holds it)
 *   then dim*max_sizes + index of the tile size                      tiles
 *   then one id                                                      bufferize (BIAS_ADD_RELU_SPLIT: one per
 *                                                                    level; mrl_rewrite.dst_level holds it)
 *   then dim*max_sizes + index of the tile size                      parallel loops
 *                                                                    (MATMUL_PARALLEL) */
typedef struct { uint8_t cls; /* 0 microkernel, 1 move, 2 tile, 3 bufferize, 4 parallel loop */
                 uint8_t operand_or_dim, dst_level, transposed, convert;
                 uint32_t tile_size, mk_index; } mrl_rewrite;
int32_t mrl_rewrite_decode(const mrl_table* tab, uint16_t id, mrl_rewrite* out);

/* shape: b,m,k,n sizes (must be in the lists); levels / layouts / dtypes: per
 * operand (FUSED: levels[4] = intermediate); entries without a coordinate are ignored.
 * The BOUNDED kinds: the memory bounds are set to their top (the capacities). */
int32_t mrl_coord_of_spec(const mrl_table* tab, const uint32_t shape[4], const uint8_t* levels,
                          const uint8_t* layouts, const uint8_t* dtypes, mrl_coord* out);

/* ---------------------------------------------------------------------------
 * Compressed table (Section 4.1, Figure 2): axis-aligned boxes [lo, hi]
 * (inclusive) of equal value that partition the lattice, sorted by lo.
 * DECISION: v0 = rewrite id, v1 = 0.  COST: the cost divided by the Spec's
 * volume b*m*k*n as a reduced fraction v0/v1; (MRL_INF, 0) for MRL_INF. */
typedef struct { uint16_t lo[MRL_MAX_DIMS], hi[MRL_MAX_DIMS]; uint64_t v0, v1; } mrl_box;
typedef enum { MRL_BOXES_DECISION = 0, MRL_BOXES_COST = 1 } mrl_box_list;

/* out: host array of cap boxes, or NULL to get the count only in *n_out. */
int32_t mrl_emit_compressed(const mrl_table* tab, uint32_t which,
                            mrl_box* out, size_t cap, size_t* n_out);

/* Point query answered from the two box lists alone (Section 4.1: the stored
 * table is the set of boxes, and a lookup finds the box that holds the Spec's
 * coordinate).  Same arguments and same answers as mrl_query, without reading
 * the dense table: the rewrite is the decision box's value, the cost is the
 * cost box's fraction times the Spec's volume.  The first call on a table
 * builds, in device memory that the library allocates and frees with the
 * table, a hierarchy of bounding boxes over each list (an R-tree bulk-loaded
 * in the list's order); the lists themselves stay in the caller's scratch
 * buffer.  Every axis must have at most 256 coordinates (MRL_E_INVAL else).
 * Errors as mrl_query. */
int32_t mrl_query_compressed(const mrl_table* tab, const mrl_coord* specs, size_t n,
                             uint64_t* cost_out, uint16_t* rewrite_out);

/* ---------------------------------------------------------------------------
 * Schedule of a goal Spec (Section 4: the search returns, for every Spec, the
 * rewrite of the cheapest implementation; following these rewrites from the
 * goal down to microkernels gives the program of Section 2, Figure 1).
 * Nodes in pre-order: a node is followed by the subtrees of its children
 * (0 for a microkernel, 1 for a tile or a Move: the loop body / the Spec on
 * the moved operand, 2 for bufferize: the Matmul, then the bias-add + ReLU;
 * in a MATMUL_CHAIN table the first Matmul, then the second, both in dep 0;
 * in a BIAS_ADD_RELU_SPLIT table the bias add, then the ReLU).
 * table: 0 = the table the walk started in, 1 + i = its dep i, 3 + i = dep i
 * of its dep 1 (a BIAS_ADD_RELU_SPLIT table read by a FUSED one); the handles
 * given to mrl_solve as deps must still be alive.  cost = the table's entry
 * of the node's Spec = cost of the whole subtree under Section 3's equation.
 * out: host array of cap nodes, or NULL to get the count only in *n_out;
 * In a MATMUL_MOVES table a Move has up to three children: the load Move Spec
 * (operands that are read), the body, the store Move Spec (the accumulated
 * output), the Move Specs in dep 0 with both tensors fresh.
 * MRL_E_INVAL if the goal has no implementation (cost MRL_INF). */
typedef struct {
  uint32_t table;
  uint16_t rewrite;
  uint16_t n_children;
  uint64_t cost;
  mrl_coord spec;
} mrl_schedule_node;
int32_t mrl_schedule(const mrl_table* tab, const mrl_coord* goal,
                     mrl_schedule_node* out, size_t cap, size_t* n_out);

/* Test support: copy the dense tables to host arrays of n_specs entries each
 * (either pointer may be NULL). */
int32_t mrl_copy_dense(const mrl_table* tab, uint64_t* cost_host, uint16_t* argmin_host);

const char* mrl_last_error(void);

#ifdef __cplusplus
}
#endif
#endif
