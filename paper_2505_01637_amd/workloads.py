"""Seeded synthetic workloads: target descriptions and spec lattices.

This module only *describes inputs* (plain Python dicts of integers).  It holds
none of the method's arithmetic: no cost formula, no admissibility rule, no
rewrite enumeration.  Both the HIP library binding and the CPU oracle binding
marshal these dicts into their own C structs.

The five configurations follow the paper's workload shapes (Section 7: the
1x2048x16384 bf16->f32 vector-matrix product and the 2048-square f32 matmul)
and its target description (Section 2.2: levels ordered RF, VRF, L1, GL;
Section 3: microkernel costs k_p, loop constant s, per-level weights).  The
paper does not print its fitted coefficients, so seeded integers stand in.
"""

MASK64 = (1 << 64) - 1
UNBOUNDED = MASK64

# microkernel kinds
MK_SCALAR_FMA = 0
MK_BCAST_VEC_MULADD = 1
MK_BF16_DOT = 2
MK_SCALAR_ADDRELU = 3
MK_VEC_ADDRELU = 4
MK_SCALAR_ADD, MK_VEC_ADD, MK_SCALAR_RELU, MK_VEC_RELU = 8, 9, 10, 11
MK_SCALAR_MOVE = 5            # Move Spec of one element (converts bf16 -> f32 if the types differ)
MK_VECTOR_MOVE = 6            # Move Spec of one row of whole vectors between level 1 and a slower level
MK_VECTOR_MOVE_ALIGNED = 7    # the same, both tensors aligned

# spec kinds
KIND_MATMUL_ACCUM = 0
KIND_BIAS_ADD_RELU = 1
KIND_FUSED_MM_ADD_RELU = 2
KIND_MATMUL_PARALLEL = 3      # a Matmul whose serial-only flag is off; reads the KIND_MATMUL_ACCUM table
KIND_MATMUL_BOUNDED = 4       # a Matmul whose Specs carry a memory bound per level of finite capacity
KIND_BIAS_ADD_RELU_BOUNDED = 5        # the same for the bias-add + ReLU
KIND_FUSED_BOUNDED = 6                # and for the fused Spec (reads the two bounded tables)
BOUNDED_KINDS = (KIND_MATMUL_BOUNDED, KIND_BIAS_ADD_RELU_BOUNDED, KIND_FUSED_BOUNDED)
KIND_MOVE = 7                 # Move Specs: source and destination tensor of rows x cols
KIND_MATMUL_MOVES = 8         # a Matmul whose Moves are Move Specs; reads a KIND_MOVE table
KIND_MATMUL_CHAIN = 9         # (lhs x rhs1) x rhs2 accumulated into out; sizes[0] holds p, the dimension the two share
KIND_BIAS_ADD = 10            # the bias add alone: in (m x n), bias (n), out (m x n)
KIND_RELU = 11                # the ReLU alone: in (m x n), out (m x n)
KIND_BIAS_ADD_RELU_SPLIT = 12 # KIND_BIAS_ADD_RELU plus a bufferize between the two; reads a KIND_BIAS_ADD and a KIND_RELU table
TWO_OPERAND_KINDS = (KIND_MOVE, KIND_RELU)
FIVE_LEVEL_KINDS = (KIND_FUSED_MM_ADD_RELU, KIND_FUSED_BOUNDED, KIND_MATMUL_CHAIN)   # four operands and an intermediate

MAX_LEVELS = 4
MAX_OPERANDS = 5


class SplitMix64:
    """Counter-based 64-bit generator (Steele, Lea, Flood 2014)."""

    def __init__(self, seed):
        self.state = seed & MASK64

    def next(self):
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)

    def draw(self, lo, hi):
        return lo + self.next() % (hi - lo + 1)


def _empty_target(n_levels, capacities):
    z3 = lambda: [[[0, 0] for _ in range(MAX_LEVELS)] for _ in range(MAX_LEVELS)]
    return {
        "n_levels": n_levels,
        "capacity_bytes": list(capacities) + [0] * (MAX_LEVELS - len(capacities)),
        "load_coef": z3(),    # [src][dst][same|transposed], dst < src
        "store_coef": z3(),   # [dst][src][same|transposed]
        "convert_coef": 0,
        "zero_coef": [0] * MAX_LEVELS,
        "loop_overhead": 0,
        "microkernels": [],   # list of (kind, lanes, cost); order = rewrite-id order
        "threads": 1,         # hardware threads of a parallel loop
        "sync_cost": 0,       # constant of a parallel loop
        "level_weight": [0] * MAX_LEVELS,   # per-level weight of a Move's cache lines (KIND_MATMUL_MOVES)
        "line_bytes": 64,     # cache line
        "strip": 0,           # columns per strip of the packed layouts (0: there are none)
    }


def _lattice(kind, sizes, layout=(0, 0, 0, 0, 0), dtype=(0, 0, 0, 0, 0),
             base_bytes=(4, 4, 4, 4, 4)):
    return {
        "kind": kind,
        "sizes": [list(s) for s in sizes],          # b, m, k, n: ascending, contain 1
        "layout_coord": list(layout),               # per operand: 0 no coordinate, 1 row-/column-major, 2 also the two packed layouts
        "dtype_coord": list(dtype),
        "base_dtype_bytes": list(base_bytes),
    }


FOUR_LEVEL_CAPS = (256, 512, 32 * 1024, UNBOUNDED)   # RF 64 f32, VRF 16x8 f32, L1 32 KiB, GL


def _four_level_target(rng):
    """Level weights grow away from RF; a Move pays weight(src)+weight(dst)."""
    t = _empty_target(4, FOUR_LEVEL_CAPS)
    w = [1, 0, 0, 0]
    for l in range(1, 4):
        w[l] = w[l - 1] + rng.draw(1, 5)
    for src in range(1, 4):
        for dst in range(src):
            t["load_coef"][src][dst][0] = w[src] + w[dst]
            t["store_coef"][dst][src][0] = w[src] + w[dst]
    t["loop_overhead"] = rng.draw(0, 4)
    t["microkernels"].append((MK_SCALAR_FMA, 1, rng.draw(1, 2)))
    t["microkernels"].append((MK_BCAST_VEC_MULADD, 8, rng.draw(1, 2)))
    return t, w


def _add_transposed(t, rng):
    for src in range(1, 4):
        for dst in range(src):
            add = rng.draw(1, 8)
            t["load_coef"][src][dst][1] = t["load_coef"][src][dst][0] + add
            t["store_coef"][dst][src][1] = t["store_coef"][dst][src][0] + add


def sizes_config4():
    return [1, 2, 4] + list(range(8, 129, 8)) + [256, 512]


def sizes_config5():
    return [1, 2, 4] + list(range(8, 257, 8)) + [512, 1024, 2048]


def config(number, seed=None, max_size=None):
    """Return {"name", "target", "lattices": [(label, lattice, dep_labels)]}.

    `max_size` drops every allowed size above it (used by tests to get a small
    lattice of the same structure); None keeps the full configuration.
    """
    rng = SplitMix64(number if seed is None else seed)
    keep = (lambda xs: [x for x in xs if max_size is None or x <= max_size])
    one = [1]
    if number == 1:
        t = _empty_target(2, (256, 32 * 1024))
        t["load_coef"][1][0][0] = rng.draw(1, 16)
        t["store_coef"][0][1][0] = rng.draw(1, 16)
        t["loop_overhead"] = rng.draw(0, 4)
        t["microkernels"].append((MK_SCALAR_FMA, 1, 1))
        r = keep(range(1, 17))
        lats = [("M", _lattice(KIND_MATMUL_ACCUM, [one, r, r, r]), [])]
    elif number == 2:
        t, _ = _four_level_target(rng)
        r = keep(range(1, 65))
        lats = [("M", _lattice(KIND_MATMUL_ACCUM, [one, r, r, r]), [])]
    elif number == 3:
        t, _ = _four_level_target(rng)
        _add_transposed(t, rng)
        t["convert_coef"] = rng.draw(1, 4)
        t["microkernels"].append((MK_BF16_DOT, 16, rng.draw(1, 2)))
        ks = keep([1 << i for i in range(12)])
        ns = keep([1 << i for i in range(15)])
        lats = [("M", _lattice(KIND_MATMUL_ACCUM, [one, one, ks, ns],
                               layout=(0, 1, 0, 0, 0), dtype=(1, 1, 0, 0, 0),
                               base_bytes=(2, 2, 4, 4, 4)), [])]
    elif number == 4:
        t, _ = _four_level_target(rng)
        _add_transposed(t, rng)
        bs = keep([1, 2, 4, 8, 16])
        r = keep(sizes_config4())
        lats = [("M", _lattice(KIND_MATMUL_ACCUM, [bs, r, r, r], layout=(1, 1, 1, 0, 0)), [])]
    elif number == 5:
        t, w = _four_level_target(rng)
        _add_transposed(t, rng)
        t["zero_coef"] = list(w)
        t["microkernels"].append((MK_SCALAR_ADDRELU, 1, 1))
        t["microkernels"].append((MK_VEC_ADDRELU, 8, 1))
        r = keep(sizes_config5())
        lats = [
            ("M", _lattice(KIND_MATMUL_ACCUM, [one, r, r, r], layout=(1, 1, 1, 0, 0)), []),
            # operands: in (m x n), bias (n), out (m x n)
            ("E", _lattice(KIND_BIAS_ADD_RELU, [one, r, one, r], layout=(1, 0, 1, 0, 0)), []),
            # operands: lhs, rhs, bias, out (+ level of the intermediate)
            ("F", _lattice(KIND_FUSED_MM_ADD_RELU, [one, r, r, r], layout=(1, 1, 0, 1, 0)),
             ["M", "E"]),
        ]
    elif number == 6:
        # beyond the five benchmark configurations: config 2's lattice twice, once serial-only
        # and once with parallel loops allowed (8 threads, a synchronisation constant well above
        # the loop constant)
        t, _ = _four_level_target(rng)
        t["threads"] = 8
        t["sync_cost"] = rng.draw(64, 256)
        r = keep(range(1, 65))
        lats = [("M", _lattice(KIND_MATMUL_ACCUM, [one, r, r, r]), []),
                ("P", _lattice(KIND_MATMUL_PARALLEL, [one, r, r, r]), ["M"])]
    elif number == 7:
        # beyond the five benchmark configurations: memory bounds as coordinates.  Four levels,
        # power-of-two sizes 1..64 on m, k, n, one bound axis per level of finite capacity
        # (RF 256 B: 10 values, VRF 512 B: 11, L1 32 KiB: 17): 343 shapes x 64 level
        # assignments x 1870 bounds = 41.0 M Specs
        t, _ = _four_level_target(rng)
        p2 = keep([1 << i for i in range(7)])
        lats = [("B", _lattice(KIND_MATMUL_BOUNDED, [one, p2, p2, p2]), [])]
    elif number == 8:
        # beyond the five benchmark configurations: config 5's three tables (Matmul, bias-add +
        # ReLU, fused) with memory bounds as coordinates, sizes 1..16 in powers of two
        t, w = _four_level_target(rng)
        _add_transposed(t, rng)
        t["zero_coef"] = list(w)
        t["microkernels"].append((MK_SCALAR_ADDRELU, 1, 1))
        t["microkernels"].append((MK_VEC_ADDRELU, 8, 1))
        p2 = keep([1 << i for i in range(5)])
        lats = [("M", _lattice(KIND_MATMUL_BOUNDED, [one, p2, p2, p2]), []),
                ("E", _lattice(KIND_BIAS_ADD_RELU_BOUNDED, [one, p2, one, p2]), []),
                ("F", _lattice(KIND_FUSED_BOUNDED, [one, p2, p2, p2]), ["M", "E"])]
    elif number == 9:
        # beyond the five benchmark configurations: Moves as Specs of their own.  Config 2's target
        # recipe; the level weights also weigh a Move's cache lines; move microkernels for one
        # element, for a row of 8-lane vectors, and (cheaper) for an aligned one.  A lattice of Move
        # Specs over sizes 1..32 (rows, columns; both layouts; contiguousness and alignment of both
        # tensors as coordinates) and the Matmul lattice over the same sizes that reads it
        t, w = _four_level_target(rng)
        t["level_weight"] = list(w)
        t["line_bytes"] = 64
        t["microkernels"].append((MK_SCALAR_MOVE, 1, rng.draw(1, 3)))
        t["microkernels"].append((MK_VECTOR_MOVE, 8, rng.draw(2, 3)))
        t["microkernels"].append((MK_VECTOR_MOVE_ALIGNED, 8, 1))
        r = keep(range(1, 33))
        lats = [("V", _lattice(KIND_MOVE, [one, r, one, r], layout=(1, 1, 0, 0, 0)), []),
                ("M", _lattice(KIND_MATMUL_MOVES, [one, r, r, r], layout=(1, 1, 1, 0, 0)), ["V"])]
    elif number == 10:
        # beyond the five benchmark configurations: the composition of two Matmuls.  Config 5's
        # target recipe (transposing Moves, initialising the intermediate); power-of-two sizes
        # 1..128 for m, k, p, n; the Matmul table over the same sizes and the lattice of
        # compositions that reads it twice (4096 shapes x 1024 level assignments x 16 layouts = 67.1 M Specs)
        t, w = _four_level_target(rng)
        _add_transposed(t, rng)
        t["zero_coef"] = list(w)
        p2 = keep([1 << i for i in range(8)])
        lats = [("M", _lattice(KIND_MATMUL_ACCUM, [one, p2, p2, p2], layout=(1, 1, 1, 0, 0)), []),
                # operands: lhs (m x k), rhs1 (k x p), rhs2 (p x n), out (m x n) (+ level of the intermediate, m x p)
                ("G", _lattice(KIND_MATMUL_CHAIN, [p2, p2, p2, p2], layout=(1, 1, 1, 1, 0)), ["M"])]
    elif number == 11:
        # beyond the five benchmark configurations: config 5's pipeline with the second bufferize.
        # Config 5's target recipe, but the vector unit has no fused add-and-ReLU: a scalar one,
        # and vector microkernels for the bias add and for the ReLU alone (and scalar ones).  The
        # bias-add + ReLU lattice S may split into the two (tables A, R), and the fused lattice
        # reads S.  Sizes: config 5's up to 256.
        t, w = _four_level_target(rng)
        _add_transposed(t, rng)
        t["zero_coef"] = list(w)
        t["microkernels"].append((MK_SCALAR_ADDRELU, 1, 1))
        t["microkernels"].append((MK_SCALAR_ADD, 1, 1))
        t["microkernels"].append((MK_VEC_ADD, 8, 1))
        t["microkernels"].append((MK_SCALAR_RELU, 1, 1))
        t["microkernels"].append((MK_VEC_RELU, 8, 1))
        r = keep([x for x in sizes_config5() if x <= 256])
        lats = [
            ("M", _lattice(KIND_MATMUL_ACCUM, [one, r, r, r], layout=(1, 1, 1, 0, 0)), []),
            ("A", _lattice(KIND_BIAS_ADD, [one, r, one, r], layout=(1, 0, 1, 0, 0)), []),
            ("R", _lattice(KIND_RELU, [one, r, one, r], layout=(1, 1, 0, 0, 0)), []),
            ("S", _lattice(KIND_BIAS_ADD_RELU_SPLIT, [one, r, one, r], layout=(1, 0, 1, 0, 0)), ["A", "R"]),
            ("F", _lattice(KIND_FUSED_MM_ADD_RELU, [one, r, r, r], layout=(1, 1, 0, 1, 0)), ["M", "S"]),
        ]
    elif number == 12:
        # beyond the five benchmark configurations: packed and shuffled layouts.  Config 9's recipe;
        # strips of 8 columns (the vector width); the Move lattice with all four layouts on both
        # tensors over sizes 1..32 (16.8 M Specs), and the Matmul lattice over the same sizes whose
        # rhs and out may be packed (lhs row- or column-major) and whose Moves are read from it
        t, w = _four_level_target(rng)
        t["level_weight"] = list(w)
        t["line_bytes"] = 64
        t["strip"] = 8
        t["microkernels"].append((MK_SCALAR_MOVE, 1, rng.draw(1, 3)))
        t["microkernels"].append((MK_VECTOR_MOVE, 8, rng.draw(2, 3)))
        t["microkernels"].append((MK_VECTOR_MOVE_ALIGNED, 8, 1))
        r = keep(range(1, 33))
        lats = [("V", _lattice(KIND_MOVE, [one, r, one, r], layout=(2, 2, 0, 0, 0)), []),
                ("M", _lattice(KIND_MATMUL_MOVES, [one, r, r, r], layout=(1, 2, 2, 0, 0)), ["V"])]
    else:
        raise ValueError("config number must be 1..12")
    return {"name": "config%d" % number, "target": t, "lattices": lats}


def n_level_axes(kind):
    return 5 if kind in FIVE_LEVEL_KINDS else 2 if kind in TWO_OPERAND_KINDS else 3


def n_operands(kind):
    return 4 if kind in FIVE_LEVEL_KINDS else 2 if kind in TWO_OPERAND_KINDS else 3


def coord_extents(target, lattice):
    """Extent of every coordinate axis: shape indices, level axes, (memory bounds,) layout bits, dtype bits."""
    kind = lattice["kind"]
    ext = [len(s) for s in lattice["sizes"]]
    ext += [target["n_levels"]] * n_level_axes(kind)
    if kind in BOUNDED_KINDS:
        # one axis per level of finite capacity: the bounds 0, 1, 2, 4, ... up to the capacity
        ext += [int(c).bit_length() + 1 for c in target["capacity_bytes"][:target["n_levels"]] if c != UNBOUNDED]
    nops = n_operands(kind)
    if kind == KIND_MOVE:
        # per tensor (source, destination): contiguousness 0..2 (0..3 where packed tensors, which
        # have three physical dimensions, exist) and the aligned flag
        nc = 4 if 2 in lattice["layout_coord"][:nops] else 3
        ext += [nc, 2, nc, 2]
    ext += [4 if lattice["layout_coord"][i] == 2 else 2 for i in range(nops) if lattice["layout_coord"][i]]
    ext += [2] * sum(1 for i in range(nops) if lattice["dtype_coord"][i])
    return ext


def n_specs(target, lattice):
    n = 1
    for e in coord_extents(target, lattice):
        n *= e
    return n
