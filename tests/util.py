"""Shared test helpers: coordinate <-> Spec conversion for the brute-force checker."""
import itertools

import numpy as np

from oracle import brute_force as B
from paper_2505_01637_amd import workloads as W


def axes(target, lattice):
    """List of (axis kind, operand) in coordinate order, and the extents."""
    kind = lattice["kind"]
    nops, nlv = W.n_operands(kind), W.n_level_axes(kind)
    ax = [("size", d) for d in range(4)] + [("level", i) for i in range(nlv)]
    if kind in W.BOUNDED_KINDS:
        ax += [("limit", l) for l in range(target["n_levels"]) if target["capacity_bytes"][l] != W.UNBOUNDED]
    if kind == W.KIND_MOVE:
        ax += [("contig", 0), ("aligned", 0), ("contig", 1), ("aligned", 1)]
    ax += [("layout", i) for i in range(nops) if lattice["layout_coord"][i]]
    ax += [("dtype", i) for i in range(nops) if lattice["dtype_coord"][i]]
    return ax, W.coord_extents(target, lattice)


def spec_of_coord(target, lattice, x):
    ax, _ = axes(target, lattice)
    dims = [1, 1, 1, 1]
    lv, ly = [0] * 5, [0] * 5
    bf = [1 if lattice["base_dtype_bytes"][i] == 2 else 0 for i in range(5)]
    lim = [None] * target["n_levels"]
    contig, aligned = [2, 2], [1, 1]
    for (what, i), v in zip(ax, x):
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


def coord_of_spec(target, lattice, spec):
    ax, _ = axes(target, lattice)
    x = []
    for what, i in ax:
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


def linear(ext, x):
    r = 0
    for e, v in zip(ext, x):
        r = r * e + v
    return r


def all_coords(ext):
    return itertools.product(*[range(e) for e in ext])


def boxes_as_tuples(boxes, ndim):
    return [(tuple(int(v) for v in b["lo"][:ndim]), tuple(int(v) for v in b["hi"][:ndim]),
             int(b["v0"]), int(b["v1"])) for b in boxes]
