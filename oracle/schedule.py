"""Schedule extraction from the oracle's tables.

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's CPU
baseline may use anything under oracle/.

Section 4 of the paper: the search memoizes, for every Spec, the rewrite of its
cheapest implementation.  Starting at a goal Spec and applying the memoized
rewrite again and again (Section 2: tile -> the loop body, Move -> the Spec on
the moved operand, bufferize -> the Matmul and the bias-add + ReLU of Section
2.1 (or the two Matmuls of a composition), microkernel -> a leaf) spells out the program of Figure 1.  The walk uses
the C oracle's dense tables for the memoized rewrites and brute_force.rewrites
for what a rewrite does to a Spec; tree_cost() evaluates Section 3's cost
equation on the result, which must give back the table's entry of the goal.
"""
from oracle import brute_force as B

INF = 2 ** 64 - 1


def axes(lattice, target=None):
    """(axis kind, operand or dimension or level) per coordinate, in coordinate order:
    sizes b, m, k, n; one level per operand (kinds F and G: plus the intermediate);
    (Move Specs: contiguousness and aligned flag of both tensors;)
    (bounded kinds: one memory bound per level of finite capacity;) layout bits; dtype bits."""
    kind = lattice["kind"]
    nops = 4 if B.base_kind(kind) in (B.F, B.G) else 2 if kind in (B.R, B.V) else 3
    nlv = 5 if B.base_kind(kind) in (B.F, B.G) else 2 if kind in (B.R, B.V) else 3
    ax = [("size", d) for d in range(4)] + [("level", i) for i in range(nlv)]
    if kind in B.BOUNDED:
        ax += [("limit", l) for l in range(target["n_levels"]) if target["capacity_bytes"][l] != INF]
    if kind == B.V:      # contiguousness and aligned flag of the source, then of the destination
        ax += [("contig", 0), ("aligned", 0), ("contig", 1), ("aligned", 1)]
    ax += [("layout", i) for i in range(nops) if lattice["layout_coord"][i]]
    ax += [("dtype", i) for i in range(nops) if lattice["dtype_coord"][i]]
    return ax


def spec_of_coord(lattice, x, target=None):
    dims = [1, 1, 1, 1]
    lv, ly = [0] * 5, [0] * 5
    bf = [1 if lattice["base_dtype_bytes"][i] == 2 else 0 for i in range(5)]
    lim = [None] * (target["n_levels"] if target else 0)
    contig, aligned = [2, 2], [1, 1]
    for (what, i), v in zip(axes(lattice, target), x):
        if what == "size":
            dims[i] = lattice["sizes"][i][v]
        elif what == "level":
            lv[i] = v
        elif what == "layout":
            ly[i] = v
        elif what == "limit":
            lim[i] = 0 if v == 0 else 1 << (v - 1)
        elif what == "contig":
            contig[i] = v
        elif what == "aligned":
            aligned[i] = v
        else:
            bf[i] = v
    return B.Spec(lattice["kind"], tuple(dims), tuple(lv), tuple(ly), tuple(bf), tuple(lim), tuple(contig), tuple(aligned))


def coord_of_spec(lattice, spec, target=None):
    x = []
    for what, i in axes(lattice, target):
        if what == "size":
            x.append(lattice["sizes"][i].index(spec.dims[i]))
        elif what == "level":
            x.append(spec.levels[i])
        elif what == "layout":
            x.append(spec.layouts[i])
        elif what == "limit":
            x.append(int(spec.limits[i]).bit_length())
        elif what == "contig":
            x.append(spec.contig[i])
        elif what == "aligned":
            x.append(spec.aligned[i])
        else:
            x.append(spec.bf16[i])
    return tuple(x)


def extract(target, lattices, results, label, coord):
    """Program tree of the Spec at `coord` of table `label`.

    lattices: [(label, lattice, dep labels)] as in workloads.config(); results:
    {label: {"cost", "argmin", "extents"}} from oracle.solve_config().  A node is
    a dict: label, coord, rewrite, cost, node (brute_force's description of the
    rewrite: tag and constants), children.  ValueError if the goal has no
    implementation."""
    by_kind = {lat["kind"]: (lab, lat) for lab, lat, _ in lattices}
    lat_of_kind = {k: v[1] for k, v in by_kind.items()}

    def walk(spec):
        lab, lat = by_kind[spec.kind]
        x = coord_of_spec(lat, spec, target)
        lin = 0
        for e, v in zip(results[lab]["extents"], x):
            lin = lin * int(e) + v
        cost, rid = int(results[lab]["cost"][lin]), int(results[lab]["argmin"][lin])
        if cost == INF:
            raise ValueError("Spec %r of table %s has no implementation" % (x, lab))
        for r, node, children in B.rewrites(target, lat_of_kind, spec):
            if r == rid:
                return {"label": lab, "coord": x, "rewrite": rid, "cost": cost, "node": node,
                        "children": [walk(ch) for ch in children]}
        raise AssertionError("the memoized rewrite %d does not apply to Spec %r" % (rid, spec))

    return walk(spec_of_coord(dict(lattices_by_label(lattices))[label], coord, target))


def lattices_by_label(lattices):
    return [(lab, lat) for lab, lat, _ in lattices]


def as_program(tree):
    """The tree in brute_force's tuple form (tag, constants..., subtrees...)."""
    return tree["node"] + tuple(as_program(ch) for ch in tree["children"])


def tree_cost(tree):
    """Section 3's cost equation evaluated on the extracted program."""
    return B.c(as_program(tree))


def preorder(tree):
    """[(label, coord, rewrite, cost, number of children)], a node before its subtrees."""
    out = [(tree["label"], tree["coord"], tree["rewrite"], tree["cost"], len(tree["children"]))]
    for ch in tree["children"]:
        out += preorder(ch)
    return out
