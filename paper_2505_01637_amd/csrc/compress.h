// Internal: host-side launchers of the kernels in fill.hip and compress.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "dev_params.h"

namespace mrl {

// Table geometry passed by value to the compression kernels (cells < 2^32).
struct Geo {
  uint32_t ndim, n;
  uint32_t ext[16], stride[16];
};

void launch_plan(const DevParams* P, uint32_t n_shapes, uint32_t npass, uint32_t G, const uint32_t* level_shapes,
                 const uint32_t* level_off, uint32_t n_levels, uint32_t* shape_class, uint32_t* list_whole,
                 uint32_t* list_slice, uint32_t* list_wide, uint32_t* list_cnt, uint32_t* fitmap, Counters* ctr,
                 void* prefill_cost, void* prefill_arg, hipStream_t stream);
void launch_fill_level(const DevParams* P, uint32_t npass, uint32_t G, uint32_t max_task, const uint32_t* list_whole,
                       uint32_t n_stretch, uint32_t n_small, uint32_t n_bigwhole, const uint32_t* list_slice,
                       uint32_t n_slice, const uint32_t* list_wide, uint32_t n_wide, uint64_t* cost, uint16_t* arg,
                       Counters* ctr, hipStream_t stream, hipStream_t wide_stream);

// Segments of one launch of the bounded fill: segment i is (dependency level of shapes, rank)
// = shapes [first_shape, first_shape + n_shapes) of the level-ordered shape list at rank[i], and
// owns workgroups [block0[i], block0[i + 1]).
constexpr uint32_t kBoundSegs = 32;
struct BoundSegs {
  uint32_t n;
  uint32_t first_shape[kBoundSegs], n_shapes[kBoundSegs], rank[kBoundSegs], block0[kBoundSegs + 1];
};
// mode 0: a lattice with memory bounds; 1: Move Specs; 2: a Matmul whose Moves are Move Specs.
void launch_fill_bounded(const DevParams* P, int mode, const uint32_t* all_level_shapes, const BoundSegs& segs, uint64_t* cost,
                         uint16_t* arg, Counters* ctr, hipStream_t stream);
void launch_fill_ones(void* p, size_t bytes, hipStream_t stream, bool short_lived = false);
void launch_zero_words(unsigned long long* p, uint32_t n, hipStream_t st);
void launch_head_flags(const Geo& g, uint32_t a0, const uint64_t* cost, const uint16_t* arg, const uint32_t* fitmap,
                       const uint32_t* axis_sizes,
                       unsigned long long* maskD, unsigned long long* maskC, unsigned long long* lineD,
                       unsigned long long* lineC, hipStream_t st);
void scan_mask_words(const unsigned long long* mask, uint32_t n_words, uint32_t* tile_tmp, uint32_t* prefix,
                     uint32_t* total, hipStream_t st);
void scan_flags(const uint8_t* flags, uint32_t n, uint32_t* tile_tmp, uint32_t* pos, uint32_t* total, hipStream_t st);
// Live boxes (alive[b]) move to dense arrays: box b becomes box pos[b].
void launch_compact_boxes(uint32_t n, const uint8_t* alive, const uint32_t* pos, const uint32_t* bcell, const void* blen,
                          uint32_t* cell2, void* len2, uint8_t* alive2, hipStream_t st);
// The first generic pass (axis a1) done on the cells, for tables whose a0 and a1 have strides of
// whole mask words with a1 outside a0 and at most 64 steps on a1: runs = the mask of pass 0,
// mask2 = runs without the heads that this pass folds into the run before them on a1, col = one
// word per column of cells along a1 (zero before), bit c set where the run at step c was folded.
void launch_second_axis(const Geo& g, uint32_t a0, uint32_t a1, bool is_cost, const unsigned long long* runs,
                        const unsigned long long* line, const uint32_t* fitmap, const uint64_t* cost, const uint16_t* arg,
                        const uint32_t* axis_sizes, unsigned long long* mask2, unsigned long long* col, hipStream_t st);
// col != nullptr: mask is launch_second_axis's mask2 and every box gets its chain's length on a1.
void launch_make_boxes(const Geo& g, uint32_t a0, const unsigned long long* mask, const uint32_t* prefix,
                       const unsigned long long* line, const unsigned long long* col, uint32_t a1, uint32_t* bcell,
                       void* blen, uint8_t* alive, hipStream_t st);
// One merge pass along axis a.  After a compaction the mask still ranks boxes by their old index:
// old_alive / remap (the compaction's alive and pos) translate it; nullptr before.
void launch_axis_pass(const Geo& g, uint32_t a, uint8_t stamp, bool is_cost, uint32_t n_boxes, const uint8_t* old_alive,
                      const uint32_t* remap, const uint32_t* bcell, void* blen, uint8_t* alive, uint32_t* next,
                      uint32_t* block_linked, const unsigned long long* mask, const uint32_t* prefix, const uint64_t* cost,
                      const uint16_t* arg, const uint32_t* axis_sizes, hipStream_t st);
// The trailing passes over axes of extent 2 whose stride is at most 32 cells, in pass order.
struct TailAxes {
  uint32_t n;
  uint32_t axis[8], stride[8];
};
void launch_tail_pairs(const TailAxes& T, bool is_cost, uint32_t n_words, const unsigned long long* mask,
                       const uint32_t* prefix, const uint8_t* old_alive, const uint32_t* remap, void* blen, uint8_t* alive,
                       const uint64_t* cost, const uint16_t* arg, hipStream_t st);
void launch_emit(const Geo& g, const DevParams* P, bool is_cost, uint32_t n_boxes, const uint32_t* bcell,
                 const void* blen,
                 const uint8_t* alive, const uint32_t* pos, const uint64_t* cost, const uint16_t* arg, uint32_t* fcell,
                 void* flen, uint64_t* fv0, uint64_t* fv1, hipStream_t st);
void launch_gather(const uint64_t* idx, uint32_t n, const uint64_t* cost, const uint16_t* arg, uint64_t* cost_out,
                   uint16_t* arg_out, hipStream_t st);

// Point lookups in a final box list: a packed hierarchy of bounding boxes over the list's order.
constexpr uint32_t kIndexFan = 8;          // children per node
constexpr uint32_t kIndexMaxLevels = 12;   // 8^11 > 2^32 boxes
struct alignas(32) BoxBounds { uint8_t lo[16], hi[16]; };   // inclusive corners, one byte per axis
struct IndexLevels {
  uint32_t n_levels;                       // level 0 = the boxes; the top level has at most kIndexFan nodes
  uint32_t count[kIndexMaxLevels], off[kIndexMaxLevels];    // nodes per level, first node of the level
  uint32_t total;
};
IndexLevels index_levels(uint32_t n_boxes);
void launch_build_index(const Geo& g, const IndexLevels& L, const uint32_t* fcell, const void* flen, BoxBounds* nodes,
                        hipStream_t st);
// points: 16 bytes per point (coordinates, zero padded).  out0/out1: the value of the box that
// holds the point; which_out: its index, 0xFFFFFFFF if none.
void launch_lookup(const Geo& g, const IndexLevels& L, const BoxBounds* nodes, const uint32_t* fcell,
                   const uint8_t* points, uint32_t n_points, const uint64_t* fv0, const uint64_t* fv1, uint64_t* out0,
                   uint64_t* out1, uint32_t* which_out, hipStream_t st);

constexpr uint32_t kScanTileItems = 2048;   // items per scan tile (tile_tmp needs n/2048 + 1 words)

}  // namespace mrl
