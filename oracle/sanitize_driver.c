/*
 * Stand-alone driver that runs the CPU oracle over a small problem read from a
 * file, so that the oracle can be built and run under
 * -fsanitize=address,undefined as an ordinary executable.
 *
 * THIS FILE IS TEST INFRASTRUCTURE, like the oracle it includes.
 *
 * Input file (native endianness, no padding between the pieces):
 *   orc_target                                  (the struct's bytes)
 *   u32 n_lattices
 *   per lattice: u32 kind; u32 n_sizes[4]; the four size lists (u32 each);
 *                u8 layout_coord[5], dtype_coord[5], base_dtype_bytes[5];
 *                i32 depM, depE                 (index of an earlier lattice, -1 = none)
 * Output file, per lattice:
 *   i32 rc; u64 n; u64 cost[n]; u16 arg[n]; u64 n_admissible, n_rewrites;
 *   u64 n_decision_boxes; orc_box[...]; u64 n_cost_boxes; orc_box[...]
 * Besides writing the results the driver checks what needs no second program:
 * both forms of the first merge pass give the same lists, and the boxes paint
 * back the dense values with every cell covered once.  Exit status 0 = all
 * checks passed (a sanitizer report ends the process with its own status).
 */
#include <stdio.h>

#include "morello_oracle.c"

enum { MAX_LATTICES = 8 };

static void need(int ok, const char* what) {
  if (!ok) { fprintf(stderr, "sanitize_driver: %s\n", what); exit(2); }
}

static void rd(FILE* f, void* p, size_t n) { need(fread(p, 1, n, f) == n, "short input file"); }
static void wr(FILE* f, const void* p, size_t n) { need(fwrite(p, 1, n, f) == n, "write failed"); }

int main(int argc, char** argv) {
  need(argc == 3, "usage: sanitize_driver <input> <output>");
  FILE* in = fopen(argv[1], "rb");
  FILE* out = fopen(argv[2], "wb");
  need(in && out, "cannot open the files");
  orc_target T;
  rd(in, &T, sizeof T);
  uint32_t n_lat;
  rd(in, &n_lat, 4);
  need(n_lat >= 1 && n_lat <= MAX_LATTICES, "bad lattice count");
  orc_lattice L[MAX_LATTICES];
  uint32_t* sizes[MAX_LATTICES][4];
  uint64_t* costs[MAX_LATTICES];
  for (uint32_t i = 0; i < n_lat; i++) {
    memset(&L[i], 0, sizeof L[i]);
    rd(in, &L[i].kind, 4);
    rd(in, L[i].n_sizes, 16);
    for (int d = 0; d < 4; d++) {
      need(L[i].n_sizes[d] >= 1 && L[i].n_sizes[d] <= 255, "bad size list");
      sizes[i][d] = (uint32_t*)malloc(L[i].n_sizes[d] * sizeof(uint32_t));
      need(sizes[i][d] != NULL, "out of memory");
      rd(in, sizes[i][d], L[i].n_sizes[d] * sizeof(uint32_t));
      L[i].sizes[d] = sizes[i][d];
    }
    rd(in, L[i].layout_coord, 5);
    rd(in, L[i].dtype_coord, 5);
    rd(in, L[i].base_dtype_bytes, 5);
    int32_t dep[2];
    rd(in, dep, 8);
    need(dep[0] < (int32_t)i && dep[1] < (int32_t)i, "a dep must be an earlier lattice");

    uint32_t ndim, ext[ORC_MAXD], order[ORC_MAXD];
    need(orc_geometry(&T, &L[i], &ndim, ext, order, NULL) == 0, "orc_geometry refused the lattice");
    uint64_t n = 1;
    for (uint32_t a = 0; a < ndim; a++) n *= ext[a];
    uint64_t* cost = (uint64_t*)malloc(n * sizeof(uint64_t));
    uint16_t* arg = (uint16_t*)malloc(n * sizeof(uint16_t));
    uint64_t* v0 = (uint64_t*)malloc(n * sizeof(uint64_t));
    uint64_t* v1 = (uint64_t*)malloc(n * sizeof(uint64_t));
    uint64_t* p0 = (uint64_t*)malloc(n * sizeof(uint64_t));
    uint64_t* p1 = (uint64_t*)malloc(n * sizeof(uint64_t));
    uint8_t* cover = (uint8_t*)malloc(n);
    need(cost && arg && v0 && v1 && p0 && p1 && cover, "out of memory");
    costs[i] = cost;
    uint64_t n_adm = 0, n_rw = 0;
    /* one goal first, so that the goal path runs as well */
    uint64_t goal = n - 1;
    int32_t rc = orc_solve(&T, &L[i], dep[0] >= 0 ? &L[dep[0]] : NULL, dep[0] >= 0 ? costs[dep[0]] : NULL,
                           dep[1] >= 0 ? &L[dep[1]] : NULL, dep[1] >= 0 ? costs[dep[1]] : NULL, &goal, 1, cost, arg,
                           &n_adm, &n_rw);
    need(rc == 0 || rc == -6, "orc_solve refused the problem");
    wr(out, &rc, 4);
    wr(out, &n, 8);
    wr(out, cost, n * sizeof(uint64_t));
    wr(out, arg, n * sizeof(uint16_t));
    wr(out, &n_adm, 8);
    wr(out, &n_rw, 8);
    for (int which = 0; which < 2; which++) {
      if (which == 0) {
        for (uint64_t x = 0; x < n; x++) { v0[x] = arg[x]; v1[x] = 0; }
      } else {
        need(orc_cost_values(&T, &L[i], cost, v0, v1) == 0, "orc_cost_values failed");
      }
      orc_box *by_lines = NULL, *by_cells = NULL;
      int64_t nb = orc_merge(ndim, ext, order, ndim, v0, v1, 1, &by_lines);
      int64_t nb2 = orc_merge(ndim, ext, order, ndim, v0, v1, 0, &by_cells);
      need(nb >= 1 && nb == nb2, "the two forms of the first merge pass give lists of different length");
      need(memcmp(by_lines, by_cells, (size_t)nb * sizeof(orc_box)) == 0, "the two forms of the first merge pass differ");
      need(orc_decompress(ndim, ext, by_lines, (uint64_t)nb, p0, p1, cover) == 0, "a box lies outside the lattice");
      for (uint64_t x = 0; x < n; x++)
        need(cover[x] == 1 && p0[x] == v0[x] && p1[x] == v1[x], "the boxes do not paint back the dense values");
      uint64_t nbu = (uint64_t)nb;
      wr(out, &nbu, 8);
      wr(out, by_lines, (size_t)nb * sizeof(orc_box));
      orc_free(by_lines);
      orc_free(by_cells);
    }
    free(arg); free(v0); free(v1); free(p0); free(p1); free(cover);
  }
  for (uint32_t i = 0; i < n_lat; i++) {
    free(costs[i]);
    for (int d = 0; d < 4; d++) free(sizes[i][d]);
  }
  fclose(in);
  need(fclose(out) == 0, "write failed");
  return 0;
}
