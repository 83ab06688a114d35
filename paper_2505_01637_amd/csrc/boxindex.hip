// Point lookups in a final box list (Section 4.1: the table is kept as boxes and a lookup finds
// the box that holds a Spec's coordinate).
//
// The boxes of a list are disjoint, cover the lattice and are sorted by their low corner in
// row-major order.  Over that order sits a packed hierarchy of bounding boxes with fan-out 8
// (level 0: the boxes themselves; a node of level l+1 bounds 8 consecutive nodes of level l),
// i.e. an R-tree bulk-loaded in the list's own order.  A lookup walks it depth first and descends
// only into nodes whose bounds contain the point; exactly one box of level 0 does.
#include <hip/hip_runtime.h>

#include "compress.h"

namespace mrl {

namespace {

__device__ __forceinline__ bool contains(const BoxBounds& b, const uint8_t* p) {
  bool in = true;
#pragma unroll
  for (int a = 0; a < 16; a++) in = in && b.lo[a] <= p[a] && p[a] <= b.hi[a];
  return in;
}

// Level 0: corners of each box from its low cell and its run lengths.  Axes beyond ndim get
// lo = hi = 0, which every point (padded with zeros) satisfies.
__global__ __launch_bounds__(256) void box_bounds_kernel(Geo g, uint32_t n, const uint32_t* __restrict__ fcell,
                                                         const uint8_t* __restrict__ flen, BoxBounds* __restrict__ out) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= n) return;
  BoxBounds b;
  uint32_t x = fcell[i];
#pragma unroll
  for (uint32_t a = 0; a < 16; a++) {
    uint32_t lo = 0, len = 1;
    if (a < g.ndim) {
      lo = x / g.stride[a];
      x -= lo * g.stride[a];
      len = flen[(size_t)i * 16 + a];
    }
    b.lo[a] = (uint8_t)lo;
    b.hi[a] = (uint8_t)(lo + len - 1);
  }
  out[i] = b;
}

__global__ __launch_bounds__(256) void group_bounds_kernel(const BoxBounds* __restrict__ in, uint32_t n_in,
                                                           BoxBounds* __restrict__ out, uint32_t n_out) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= n_out) return;
  BoxBounds r;
#pragma unroll
  for (int a = 0; a < 16; a++) { r.lo[a] = 255; r.hi[a] = 0; }
  const uint32_t first = i * kIndexFan;
  const uint32_t last = min(first + kIndexFan, n_in);
  for (uint32_t c = first; c < last; c++) {
    const BoxBounds b = in[c];
#pragma unroll
    for (int a = 0; a < 16; a++) {
      r.lo[a] = min(r.lo[a], b.lo[a]);
      r.hi[a] = max(r.hi[a], b.hi[a]);
    }
  }
  out[i] = r;
}

// One lane per point.  The boxes are sorted by low corner in row-major order and the box that
// holds a point starts at or before the point in that order, so the walk starts at the last box
// whose low cell is <= the point's cell (binary search) and runs backwards: the box wanted is
// usually a few boxes away.  cursor/first: the stretch of nodes still to test on each level,
// taken from its end; every node is tested at most once, so the walk ends.  which_out: the
// box's index, or 0xFFFFFFFF if no box holds the point (the list is then not a partition:
// reported by the host).
__global__ __launch_bounds__(256) void lookup_kernel(Geo g, IndexLevels L, const BoxBounds* __restrict__ nodes,
                                                     const uint32_t* __restrict__ fcell,
                                                     const uint8_t* __restrict__ points, uint32_t n_points,
                                                     const uint64_t* __restrict__ fv0, const uint64_t* __restrict__ fv1,
                                                     uint64_t* __restrict__ out0, uint64_t* __restrict__ out1,
                                                     uint32_t* __restrict__ which_out) {
  const uint32_t q = blockIdx.x * 256u + threadIdx.x;
  if (q >= n_points) return;
  uint8_t p[16];
  uint32_t cell = 0;
#pragma unroll
  for (int a = 0; a < 16; a++) {
    p[a] = points[(size_t)q * 16 + a];
    if ((uint32_t)a < g.ndim) cell += p[a] * g.stride[a];
  }
  // pos = number of boxes whose low cell is <= cell (>= 1 for a partition: box 0 starts at cell 0)
  uint32_t lo = 0, hi = L.count[0];
  while (lo < hi) {
    const uint32_t mid = lo + (hi - lo) / 2;
    if (fcell[mid] <= cell) lo = mid + 1; else hi = mid;
  }
  uint32_t found = 0xFFFFFFFFu;
  if (lo > 0) {
    const uint32_t pos = lo - 1;
    // cursor[l]: one past the next node to test on level l; first[l]: where its stretch begins
    uint32_t cursor[kIndexMaxLevels], first[kIndexMaxLevels];
    int lvl = (int)L.n_levels - 1;
    cursor[lvl] = (pos >> (3 * lvl)) + 1;
    first[lvl] = 0;
    while (true) {
      if (cursor[lvl] == first[lvl]) {
        if (lvl == (int)L.n_levels - 1) break;
        lvl++;
        continue;
      }
      const uint32_t i = --cursor[lvl];
      if (!contains(nodes[L.off[lvl] + i], p)) continue;
      if (lvl == 0) { found = i; break; }
      lvl--;
      first[lvl] = i * kIndexFan;
      cursor[lvl] = min(i * kIndexFan + kIndexFan, (pos >> (3 * lvl)) + 1);
    }
  }
  which_out[q] = found;
  out0[q] = found == 0xFFFFFFFFu ? 0 : fv0[found];
  out1[q] = found == 0xFFFFFFFFu ? 0 : fv1[found];
}

}  // namespace

IndexLevels index_levels(uint32_t n_boxes) {
  IndexLevels L;
  L.n_levels = 0;
  L.total = 0;
  uint32_t n = n_boxes;
  while (true) {
    L.count[L.n_levels] = n;
    L.off[L.n_levels] = L.total;
    L.total += n;
    L.n_levels++;
    if (n <= kIndexFan || L.n_levels == kIndexMaxLevels) break;
    n = (n + kIndexFan - 1) / kIndexFan;
  }
  return L;
}

void launch_build_index(const Geo& g, const IndexLevels& L, const uint32_t* fcell, const void* flen, BoxBounds* nodes,
                        hipStream_t st) {
  const uint32_t n = L.count[0];
  if (!n) return;
  hipLaunchKernelGGL(box_bounds_kernel, dim3((n + 255) / 256), dim3(256), 0, st, g, n, fcell, (const uint8_t*)flen, nodes);
  for (uint32_t l = 1; l < L.n_levels; l++)
    hipLaunchKernelGGL(group_bounds_kernel, dim3((L.count[l] + 255) / 256), dim3(256), 0, st, nodes + L.off[l - 1],
                       L.count[l - 1], nodes + L.off[l], L.count[l]);
}

void launch_lookup(const Geo& g, const IndexLevels& L, const BoxBounds* nodes, const uint32_t* fcell,
                   const uint8_t* points, uint32_t n_points, const uint64_t* fv0, const uint64_t* fv1, uint64_t* out0,
                   uint64_t* out1, uint32_t* which_out, hipStream_t st) {
  if (!n_points) return;
  static_assert(kIndexFan == 8, "the walk shifts box indices by 3 bits per level");
  hipLaunchKernelGGL(lookup_kernel, dim3((n_points + 255) / 256), dim3(256), 0, st, g, L, nodes, fcell, points, n_points,
                     fv0, fv1, out0, out1, which_out);
}

}  // namespace mrl
