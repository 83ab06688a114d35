"""Exhaustive schedule enumeration and an explicit program-tree cost evaluator.

TEST INFRASTRUCTURE, written separately from the C oracle so that the two can
be checked against each other on tiny lattices.

* `programs(...)` walks the rewrites of Section 2 (tile, move, select) and
  Section 2.1 (bufferize) and yields every *complete* program tree reachable
  from a Spec -- no memo table, no pruning, no cost bookkeeping.
* `c(p)` evaluates the cost equation of Section 3 on such a tree:
    loop          trips * c(body) + s
    parallel loop ceil(trips / threads) * c(body) + s_parallel
    pipeline      sum of the children (+ the intermediate's initialisation)
    alloc-binding move cost + c(children): the body, and where Moves are Specs the load and store
    microkernel   k_p
* `optimum(...)` = the minimum of c over all programs, and the lowest rewrite
  id among the first rewrites that reach it.

Only usable on very small lattices: the number of programs grows
exponentially with the number of divisors and levels.
"""
from collections import namedtuple

M, E, F, P = 0, 1, 2, 3      # P: a Matmul that may use parallel loops; M is serial-only
BD, BE, BF = 4, 5, 6          # M, E, F whose Specs carry per-level memory bounds (Sections 2.2, 2.4.4)
V, MV = 7, 8                  # V: Move Specs (Section 2.2); MV: a Matmul whose Moves are Move Specs
G = 9                         # two composed Matmuls (Section 2.1): dims = (p, m, k, n); lhs m x k, rhs1 k x p, rhs2 p x n, out m x n
A, R, S = 10, 11, 12          # bias add alone; ReLU alone; bias add -> ReLU with the bufferize between the two (Section 2.1)
BOUNDED = (BD, BE, BF)
MATMULS = (M, P, BD, MV)


def base_kind(kind):
    """The operator of a kind: M for the Matmuls, E, F, V."""
    return M if kind in MATMULS else E if kind in (E, BE, S) else kind if kind in (V, G, A, R) else F
FMA, BCAST, BF16DOT, S_ADDRELU, V_ADDRELU = 0, 1, 2, 3, 4
S_MOVE, V_MOVE, V_MOVE_ALIGNED = 5, 6, 7
S_ADD, V_ADD, S_RELU, V_RELU = 8, 9, 10, 11

# dims = (b, m, k, n) actual sizes; levels per operand (F: 5th = intermediate);
# layouts / bf16 per operand (0 where the lattice has no such coordinate)
# limits (kind BD): bytes a program may still allocate per level, None = unbounded level
# contig / aligned (kind V): per tensor (source, destination) the abstract values of Section 2.4.3
Spec = namedtuple("Spec", "kind dims levels layouts bf16 limits contig aligned", defaults=((), (), ()))


def operand_numel(spec, i):
    b, m, k, n = spec.dims
    if spec.kind in MATMULS:
        return (b * m * k, b * k * n, b * m * n)[i]
    if base_kind(spec.kind) in (E, A):
        return (m * n, n, m * n)[i]
    if spec.kind in (V, R):
        return m * n
    if spec.kind == G:
        p = b
        return (m * k, k * p, p * n, m * n, m * p)[i]
    return (m * k, k * n, n, m * n, m * n)[i]


def operand_mode(kind, i):
    """'r' read, 'rw' accumulate, 'w' write-only."""
    if kind in MATMULS:
        return "rw" if i == 2 else "r"
    if base_kind(kind) in (E, A):
        return "w" if i == 2 else "r"
    if kind == R:
        return "w" if i == 1 else "r"
    if kind == G:
        return "rw" if i == 3 else "r"     # the second Matmul accumulates
    return "w" if i == 3 else "r"


def physical_dims(target, layout, rows, cols):
    """Extents of the physical dimensions, outermost first (Section 2.4.2): row-major, column-major,
    and for the two packed layouts strips, rows, columns of a strip."""
    if layout == 0:
        return (rows, cols)
    if layout == 1:
        return (cols, rows)
    s = target["strip"]
    if cols >= s:
        return (cols // s, rows, s)
    return (1, rows, cols)            # a tile out of one strip: the same part of every row of the strip


def most_adjacent(target, layout, cols):
    """Upper limit of contiguousness: all physical dimensions of a tensor of whole strips (or of a
    row-/column-major one); of a part of a strip only the part itself (rows lie a strip apart),
    and of a shuffled strip not even that, unless the part is one column."""
    if layout < 2:
        return 2
    if cols >= target["strip"]:
        return 3
    if layout == 2:
        return 1
    return 1 if cols == 1 else 0


def tensor_exists(target, spec, i):
    b, m, k, n = spec.dims
    rows, cols = (m, n) if spec.kind == V else ((m, k), (k, n), (m, n))[i]
    if spec.layouts[i] >= 2:
        s = target["strip"]
        whole_strips = cols % s == 0
        part_of_one = cols < s and s % cols == 0
        if not (whole_strips or (part_of_one and spec.kind == V)):      # an operand of a Matmul is a whole tensor
            return False
    if spec.kind == V and spec.contig[i] > most_adjacent(target, spec.layouts[i], cols):
        return False
    return True


def fits(target, spec):
    if spec.kind in (V, MV) and not all(tensor_exists(target, spec, i) for i in range(2 if spec.kind == V else 3)):
        return False
    if spec.kind in BOUNDED or spec.kind == V:
        return True          # the bounds decide at each allocation, not the operands' footprint;
                             # the two tensors of a Move exist already
    used = [0] * target["n_levels"]
    nops = 4 if spec.kind in (F, G) else 2 if spec.kind == R else 3
    for i in range(nops):
        used[spec.levels[i]] += operand_numel(spec, i) * (2 if spec.bf16[i] else 4)
    if spec.kind in (F, G):
        used[spec.levels[4]] += 4 * operand_numel(spec, 4)
    return all(u <= cap for u, cap in zip(used, target["capacity_bytes"]))


def microkernel_reps(target, lattice, spec, j):
    kind, lanes, _ = target["microkernels"][j]
    b, m, k, n = spec.dims
    lv, ly, bf = spec.levels, spec.layouts, spec.bf16
    if kind == FMA:
        ok = spec.kind in MATMULS and (b, m, k, n) == (1, 1, 1, 1) and tuple(lv[:3]) == (0, 0, 0) and not any(bf[:3])
        return 1 if ok else 0
    if kind == BCAST:
        rowlike = lambda y: y == 0 or (y == 2 and target["strip"] % lanes == 0)   # one row in whole strips reads like a row
        ok = (spec.kind in MATMULS and (b, m, k) == (1, 1, 1) and n % lanes == 0
              and tuple(lv[:3]) == (0, 1, 1) and not any(bf[:3]) and rowlike(ly[1]) and rowlike(ly[2]))
        return n // lanes if ok else 0
    if kind == BF16DOT:
        rhs_col = ly[1] == 1 or not lattice["layout_coord"][1]
        ok = (spec.kind in MATMULS and (b, m, n) == (1, 1, 1) and k % lanes == 0
              and tuple(lv[:3]) == (1, 1, 0) and bf[0] and bf[1] and not bf[2] and rhs_col)
        return k // lanes if ok else 0
    if kind == S_ADDRELU:
        ok = base_kind(spec.kind) == E and (m, n) == (1, 1) and tuple(lv[:3]) == (0, 0, 0)
        return 1 if ok else 0
    if kind == V_ADDRELU:
        ok = (base_kind(spec.kind) == E and m == 1 and n % lanes == 0 and tuple(lv[:3]) == (1, 1, 1)
              and ly[0] == 0 and ly[2] == 0)
        return n // lanes if ok else 0
    if kind == S_ADD:
        ok = spec.kind == A and (m, n) == (1, 1) and tuple(lv[:3]) == (0, 0, 0)
        return 1 if ok else 0
    if kind == V_ADD:
        ok = spec.kind == A and m == 1 and n % lanes == 0 and tuple(lv[:3]) == (1, 1, 1) and ly[0] == 0 and ly[2] == 0
        return n // lanes if ok else 0
    if kind == S_RELU:
        ok = spec.kind == R and (m, n) == (1, 1) and tuple(lv[:2]) == (0, 0)
        return 1 if ok else 0
    if kind == V_RELU:
        ok = spec.kind == R and m == 1 and n % lanes == 0 and tuple(lv[:2]) == (1, 1) and ly[0] == 0 and ly[1] == 0
        return n // lanes if ok else 0
    if kind == S_MOVE:
        ok = spec.kind == V and (m, n) == (1, 1) and not (bf[1] and not bf[0])
        return 1 if ok else 0
    if kind in (V_MOVE, V_MOVE_ALIGNED):
        ok = (spec.kind == V and m == 1 and n % lanes == 0
              and ((lv[0] == 1 and lv[1] > 1) or (lv[1] == 1 and lv[0] > 1))
              and all(y == 0 or (y >= 2 and (n < target["strip"] or target["strip"] % lanes == 0)) for y in ly[:2])
              and (ly[0] == 3) == (ly[1] == 3) and bf[0] == bf[1]
              and spec.contig[0] >= 1 and spec.contig[1] >= 1
              and (kind == V_MOVE or (spec.aligned[0] and spec.aligned[1])))
        return n // lanes if ok else 0
    return 0


def tiled_tensor(target, spec, t, rows2, cols2):
    """(contiguousness, aligned) of tensor t of a Move Spec after cutting a rows2 x cols2 tile out
    of it (Section 2.4.3)."""
    rows, cols = spec.dims[1], spec.dims[3]
    if spec.layouts[t] >= 2:
        s = target["strip"]
        for cc in (cols, cols2):
            if not (cc % s == 0 or (cc < s and s % cc == 0)):
                return 0, 0                 # no such tensor, or no such tile: the sub-Spec has no program anyway
    whole = physical_dims(target, spec.layouts[t], rows, cols)
    part = physical_dims(target, spec.layouts[t], rows2, cols2)
    e = 2 if spec.bf16[t] else 4
    line = target["line_bytes"]
    uncut = 0           # innermost dimensions that the tile takes whole
    for w, p in zip(reversed(whole), reversed(part)):
        if w != p:
            break
        uncut += 1
    contig = min(spec.contig[t], 1 + uncut, most_adjacent(target, spec.layouts[t], cols2))
    suffixes, prod = [], e
    for p in reversed(part):
        prod *= p
        suffixes.append(prod)
    part_of_strip = spec.layouts[t] >= 2 and cols2 < target["strip"]      # not known to be aligned
    aligned = int(bool(spec.aligned[t]) and spec.contig[t] == len(whole) and not part_of_strip
                  and all(x % line == 0 for x in suffixes))
    return contig, aligned


def cache_lines(target, elems, nbytes):
    return -(-(elems * nbytes) // target["line_bytes"])


def rewrites(target, lattices, spec):
    """Yield (rewrite_id, node_without_children, [child specs]) for every
    applicable rewrite of an admissible Spec, ids ascending."""
    lattice = lattices[spec.kind]
    nl = target["n_levels"]
    nops = 4 if base_kind(spec.kind) in (F, G) else 2 if spec.kind in (V, R) else 3
    nmk = len(target["microkernels"])
    maxs = max(len(s) for s in lattice["sizes"])
    move_base = nmk
    xw = 4 if 2 in lattice["layout_coord"][:nops] else 2       # layout changes a Move id can name
    tile_base = nmk + nops * (nl - 1) * 2 * xw
    for j in range(nmk):
        reps = microkernel_reps(target, lattice, spec, j)
        if reps:
            yield j, ("mk", target["microkernels"][j][2] * reps), []
    for i in range(0 if spec.kind == V else nops):
        mode = operand_mode(spec.kind, i)
        src = spec.levels[i]
        for dst in range(src):
            for x in range(xw):
                for cv in (0, 1):
                    if x and not lattice["layout_coord"][i]:
                        continue
                    if x >= 2 and lattice["layout_coord"][i] != 2:
                        continue
                    if cv and not (lattice["dtype_coord"][i] and spec.bf16[i] and mode == "r"):
                        continue
                    if spec.kind == MV:
                        # Section 2, Memory Movement: load Move Spec (unless only written), body, store
                        # Move Spec (if written); Section 3: m(src) + m(dest) on top of the children
                        b_, m_, k_, n_ = spec.dims
                        rows, cols = ((m_, k_), (k_, n_), (m_, n_))[i]
                        y0, y1 = spec.layouts[i], spec.layouts[i] ^ x
                        f0, f1 = spec.bf16[i], 0 if cv else spec.bf16[i]
                        top = dict(kind=V, dims=(1, rows, 1, cols), limits=(), aligned=(1, 1))
                        n0 = 3 if y0 >= 2 else 2        # fresh tensors: every physical dimension adjacent
                        n1 = 3 if y1 >= 2 else 2
                        kids = []
                        if "r" in mode:
                            kids.append(Spec(levels=(src, dst), layouts=(y0, y1), bf16=(f0, f1), contig=(n0, n1), **top))
                        lv = list(spec.levels); lv[i] = dst
                        ly = list(spec.layouts); ly[i] = y1
                        bf = list(spec.bf16); bf[i] = f1
                        kids.append(spec._replace(levels=tuple(lv), layouts=tuple(ly), bf16=tuple(bf)))
                        if "w" in mode:
                            kids.append(Spec(levels=(dst, src), layouts=(y1, y0), bf16=(f1, f0), contig=(n1, n0), **top))
                        w = target["level_weight"]
                        fixed = (cache_lines(target, rows * cols, 2 if f0 else 4) * w[src]
                                 + cache_lines(target, rows * cols, 2 if f1 else 4) * w[dst])
                        rid = move_base + ((i * (nl - 1) + dst) * xw + x) * 2 + cv
                        yield rid, ("alloc", fixed), kids
                        continue
                    coef = 0
                    if "r" in mode:
                        if target["load_coef"][src][dst][x] == 0:
                            continue
                        coef += target["load_coef"][src][dst][x]
                    if "w" in mode:
                        if target["store_coef"][dst][src][x] == 0:
                            continue
                        coef += target["store_coef"][dst][src][x]
                    if cv:
                        coef += target["convert_coef"]
                    lv = list(spec.levels); lv[i] = dst
                    ly = list(spec.layouts); ly[i] ^= x
                    bf = list(spec.bf16)
                    if cv:
                        bf[i] = 0
                    child = spec._replace(levels=tuple(lv), layouts=tuple(ly), bf16=tuple(bf))
                    if spec.kind in BOUNDED and spec.limits[dst] is not None:
                        # the buffer in dst comes out of dst's bound; what is left is rounded
                        # down to a power of two (or is zero)
                        need = operand_numel(spec, i) * (2 if bf[i] else 4)
                        if need > spec.limits[dst]:
                            continue
                        left = spec.limits[dst] - need
                        lim = list(spec.limits)
                        lim[dst] = 0 if left == 0 else 1 << (left.bit_length() - 1)
                        child = child._replace(limits=tuple(lim))
                    rid = move_base + ((i * (nl - 1) + dst) * xw + x) * 2 + cv
                    yield rid, ("alloc", coef * operand_numel(spec, i)), [child]
    for d in range(4):
        if base_kind(spec.kind) != M and d in (0, 2):
            continue
        cur = spec.dims[d]
        for j, t in enumerate(lattice["sizes"][d]):
            if t < cur and cur % t == 0:
                dims = list(spec.dims); dims[d] = t
                child = spec._replace(dims=tuple(dims))
                if spec.kind == V:
                    pairs = [tiled_tensor(target, spec, ts, dims[1], dims[3]) for ts in (0, 1)]
                    child = child._replace(contig=tuple(p[0] for p in pairs), aligned=tuple(p[1] for p in pairs))
                yield (tile_base + d * maxs + j,
                       ("loop", cur // t, target["loop_overhead"]),
                       [child])
    if spec.kind == P:
        # the body of a parallel loop is serial-only: the same Spec in the serial lattice
        for d in (0, 1, 3):
            cur = spec.dims[d]
            for j, t in enumerate(lattice["sizes"][d]):
                if t < cur and cur % t == 0:
                    dims = list(spec.dims); dims[d] = t
                    yield (tile_base + 4 * maxs + 1 + d * maxs + j,
                           ("parallel", cur // t, target["threads"], target["sync_cost"]),
                           [spec._replace(kind=M, dims=tuple(dims))])
    if base_kind(spec.kind) == F:
        b, m, k, n = spec.dims
        l_lhs, l_rhs, l_bias, l_out, l_mid = spec.levels
        y_lhs, y_rhs, _, y_out = spec.layouts[:4]
        bounded = spec.kind == BF
        lim = spec.limits
        if bounded and lim[l_mid] is not None:
            # the intermediate (m x n, f32) comes out of its level's bound; both stages get the rest
            need = 4 * m * n
            if need > lim[l_mid]:
                return
            left = lim[l_mid] - need
            lim = list(lim)
            lim[l_mid] = 0 if left == 0 else 1 << (left.bit_length() - 1)
            lim = tuple(lim)
        mm = Spec(BD if bounded else M, (1, m, k, n), (l_lhs, l_rhs, l_mid, 0, 0), (y_lhs, y_rhs, 0, 0, 0), (0,) * 5, lim)
        # (the second stage is a Spec of whichever bias-add + ReLU lattice is there: kind E, or kind S with its own bufferize)
        ee = Spec(BE if bounded else S if S in lattices else E, (1, m, 1, n), (l_mid, l_bias, l_out, 0, 0), (0, 0, y_out, 0, 0), (0,) * 5, lim)
        yield tile_base + 4 * maxs, ("pipeline", target["zero_coef"][l_mid] * m * n), [mm, ee]


    if spec.kind == S:
        # bufferize(l): the bias add writes the intermediate (m x n, f32, row-major) in level l, the
        # ReLU reads it; the intermediate must fit level l next to the operands that live there
        b, m, k, n = spec.dims
        l_in, l_bias, l_out = spec.levels[:3]
        for l in range(nl):
            used = 4 * m * n + sum(4 * operand_numel(spec, i) for i in range(3) if spec.levels[i] == l)
            if used > target["capacity_bytes"][l]:
                continue
            add = Spec(A, (1, m, 1, n), (l_in, l_bias, l, 0, 0), (spec.layouts[0], 0, 0, 0, 0), (0,) * 5)
            relu = Spec(R, (1, m, 1, n), (l, l_out, 0, 0, 0), (0, spec.layouts[2], 0, 0, 0), (0,) * 5)
            yield tile_base + 4 * maxs + l, ("pipeline", 0), [add, relu]
    if spec.kind == G:
        p, m, k, n = spec.dims
        l_lhs, l_rhs1, l_rhs2, l_out, l_mid = spec.levels
        y_lhs, y_rhs1, y_rhs2, y_out = spec.layouts[:4]
        first = Spec(M, (1, m, k, p), (l_lhs, l_rhs1, l_mid, 0, 0), (y_lhs, y_rhs1, 0, 0, 0), (0,) * 5)
        second = Spec(M, (1, m, p, n), (l_mid, l_rhs2, l_out, 0, 0), (0, y_rhs2, y_out, 0, 0), (0,) * 5)
        yield tile_base + 4 * maxs, ("pipeline", target["zero_coef"][l_mid] * m * p), [first, second]


def programs(target, lattices, spec):
    """Yield (first_rewrite_id, tree) for every complete program of `spec`."""
    if not fits(target, spec):
        return
    for rid, node, children in rewrites(target, lattices, spec):
        if not children:
            yield rid, node
        elif len(children) == 1:
            for _, sub in programs(target, lattices, children[0]):
                yield rid, node + (sub,)
        elif len(children) == 2:
            for _, pa in programs(target, lattices, children[0]):
                for _, pb in programs(target, lattices, children[1]):
                    yield rid, node + (pa, pb)
        else:
            for _, pa in programs(target, lattices, children[0]):
                for _, pb in programs(target, lattices, children[1]):
                    for _, pc in programs(target, lattices, children[2]):
                        yield rid, node + (pa, pb, pc)


def c(p):
    tag = p[0]
    if tag == "mk":
        return p[1]
    if tag == "loop":
        return p[1] * c(p[3]) + p[2]
    if tag == "parallel":
        trips, threads, sync = p[1], p[2], p[3]
        return -(-trips // threads) * c(p[4]) + sync
    if tag == "alloc":
        return p[1] + sum(c(q) for q in p[2:])
    if tag == "pipeline":
        return p[1] + c(p[2]) + c(p[3])
    raise ValueError(tag)


def optimum(target, lattices, spec):
    """(min cost, lowest first-rewrite id reaching it, number of programs); (None, None, 0) if none."""
    best = None
    arg = None
    count = 0
    for rid, tree in programs(target, lattices, spec):
        count += 1
        v = c(tree)
        if best is None or v < best or (v == best and rid < arg):
            best, arg = v, rid
    return best, arg, count


def count_rewrites(target, lattices, spec):
    """Number of rewrites enumerated for one Spec (0 when it does not fit)."""
    if not fits(target, spec):
        return 0
    return sum(1 for _ in rewrites(target, lattices, spec))


def merge_boxes(ext, merge_order, values):
    """Box merge of Section 4.1 written with dictionaries: `values` maps each
    coordinate tuple to a hashable value.  For every axis in turn, boxes that
    agree in value and in their extent on all other axes are chained when one
    starts right after the other ends.  Returns [(lo, hi, value)] sorted by lo."""
    boxes = [(x, x, v) for x, v in values.items()]
    for a in merge_order:
        groups = {}
        for lo, hi, v in boxes:
            key = (v, lo[:a] + lo[a + 1:], hi[:a] + hi[a + 1:])
            groups.setdefault(key, []).append((lo, hi))
        boxes = []
        for (v, _, _), members in groups.items():
            members.sort(key=lambda b: b[0][a])
            cur_lo, cur_hi = members[0]
            for lo, hi in members[1:]:
                if lo[a] == cur_hi[a] + 1:
                    cur_hi = hi
                else:
                    boxes.append((cur_lo, cur_hi, v))
                    cur_lo, cur_hi = lo, hi
            boxes.append((cur_lo, cur_hi, v))
    boxes.sort(key=lambda b: b[0])
    return boxes
