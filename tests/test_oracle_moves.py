"""Pins of the oracle's Move lattice (Section 2.2: Moves are Specs of their own; Section 2.4.3:
contiguousness and alignment as abstract values of a tensor specification) and of the Matmul
lattice whose alloc-bindings hold Move Specs and cost m(src) + m(dest) (Section 2, Memory
Movement; Section 3)."""
import numpy as np
import pytest

from oracle import brute_force as B
from oracle import oracle as O
from paper_2505_01637_amd import workloads as W

import util
from test_oracle_pins import brute_force_compare


def move_target(line_bytes=8, s=1, scalar=3, vec=2, vec_aligned=1, lanes=2):
    """Three levels: registers, vector registers, memory.  A cache line of 8 bytes, so that
    alignment and whole lines matter already for tensors of a few elements."""
    t = W._empty_target(3, (64, 128, W.UNBOUNDED))
    t["loop_overhead"] = s
    t["line_bytes"] = line_bytes
    t["level_weight"] = [1, 2, 5, 0]
    t["microkernels"] = [(W.MK_SCALAR_MOVE, 1, scalar), (W.MK_VECTOR_MOVE, lanes, vec),
                         (W.MK_VECTOR_MOVE_ALIGNED, lanes, vec_aligned)]
    return t


def move_lattice(sizes, layout=(1, 1), dtype=(1, 1)):
    return W._lattice(W.KIND_MOVE, [[1], list(sizes), [1], list(sizes)], layout=layout + (0, 0, 0), dtype=dtype + (0, 0, 0))


def test_brute_force_move_lattice():
    """Every Spec of a small Move lattice (sizes 1, 2, 4; three levels; both layouts, both types,
    every contiguousness and alignment value) against the minimum over all complete programs."""
    t = move_target()
    lats = [("V", move_lattice([1, 2, 4]), [])]
    res = O.solve_config({"target": t, "lattices": lats})
    assert res["V"]["extents"] == [1, 3, 1, 3, 3, 3, 3, 2, 3, 2, 2, 2, 2, 2]
    n = brute_force_compare(t, lats, res, "V")
    assert n == len(res["V"]["cost"]) == 46656
    assert res["V"]["n_admissible"] == n


def test_move_lattice_closed_forms():
    t = move_target(s=0)
    lat = move_lattice([1, 2, 4, 8])
    ext = W.coord_extents(t, lat)
    c = O.solve(t, lat)["cost"].reshape(ext)
    a = O.solve(t, lat)["argmin"].reshape(ext)
    i = {1: 0, 2: 1, 4: 2, 8: 3}
    top = (2, 1, 2, 1)            # both tensors contiguous and aligned
    # a row of whole lines from memory into vector registers, f32, row-major: aligned vector moves, one per 2 lanes
    for cols in (2, 4, 8):
        assert int(c[(0, 0, 0, i[cols], 2, 1) + top + (0, 0, 0, 0)]) == cols // 2 * 1
        assert int(a[(0, 0, 0, i[cols], 2, 1) + top + (0, 0, 0, 0)]) == 2           # select(VECTOR_MOVE_ALIGNED)
        # the store is the same Spec the other way round
        assert int(c[(0, 0, 0, i[cols], 1, 2) + top + (0, 0, 0, 0)]) == cols // 2 * 1
        # not known to be aligned: the plain vector move
        assert int(c[(0, 0, 0, i[cols], 2, 1, 2, 0, 2, 1, 0, 0, 0, 0)]) == cols // 2 * 2
        # values not adjacent in the source: element by element (a loop over columns, no loop constant here)
        assert int(c[(0, 0, 0, i[cols], 2, 1, 0, 1, 2, 1, 0, 0, 0, 0)]) == cols * 3
    # 4 x 8 f32, no loop constant: 4 rows of 32 bytes, every row a whole number of 8-byte lines, so the
    # rows stay aligned (Section 2.4.3: aligned, contiguous, and every suffix a multiple of the line)
    assert int(c[(0, i[4], 0, i[8], 2, 1) + top + (0, 0, 0, 0)]) == 4 * 4 * 1
    # bf16: a row of 2 elements is 4 bytes, half a line: its tiles are not known to be aligned
    assert int(c[(0, i[4], 0, i[2], 2, 1) + top + (0, 0, 1, 1)]) == 4 * 1 * 2
    # column-major tensors: no vector move takes them (their rows are not the inner dimension): scalar moves
    assert int(c[(0, 0, 0, i[4], 2, 1) + top + (1, 1, 0, 0)]) == 4 * 3
    # a conversion is element by element as well, and narrowing does not exist
    assert int(c[(0, 0, 0, i[4], 2, 1) + top + (0, 0, 1, 0)]) == 4 * 3
    assert int(c[(0, 0, 0, i[4], 2, 1) + top + (0, 0, 0, 1)]) == O.INF
    # between registers and vector registers there is no vector move (one side must be slower than level 1)
    assert int(c[(0, 0, 0, i[4], 1, 0) + top + (0, 0, 0, 0)]) == 4 * 3


def test_move_lattice_invariants():
    """Knowing more never hurts: the cost does not rise with contiguousness or with alignment.
    Filling from other goals first gives the same table."""
    t = move_target()
    lat = move_lattice([1, 2, 4, 8])
    ext = W.coord_extents(t, lat)
    r = O.solve(t, lat)
    c = r["cost"].reshape(ext)
    for axis in (6, 7, 8, 9):
        x = np.moveaxis(c, axis, 0)
        assert (x[1:] <= x[:-1]).all()
    assert (c[:, :, :, :, :, :, 0] > c[:, :, :, :, :, :, 2]).any()
    assert (c[:, :, :, :, :, :, :, 0] > c[:, :, :, :, :, :, :, 1]).any()
    goals = np.random.default_rng(3).permutation(len(r["cost"]))[:500]
    again = O.solve(t, lat, goals=goals)
    assert np.array_equal(again["cost"], r["cost"]) and np.array_equal(again["argmin"], r["argmin"])
    assert again["n_rewrites"] == r["n_rewrites"]


def matmul_with_moves(sizes, levels=3, layout=(0, 0, 0), dtype=(0, 0, 0), base=(4, 4, 4), **kw):
    t = move_target(**kw)
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 1)] + t["microkernels"]
    if levels == 2:
        t["n_levels"] = 2
        t["capacity_bytes"] = [64, W.UNBOUNDED, 0, 0]
    any_lay, any_dt = any(layout), any(dtype) or 2 in base
    lats = [("V", move_lattice(sizes, layout=(1, 1) if any_lay else (0, 0), dtype=(1, 1) if any_dt else (0, 0)), []),
            ("M", W._lattice(W.KIND_MATMUL_MOVES, [[1], list(sizes), list(sizes), list(sizes)],
                             layout=tuple(layout) + (0, 0), dtype=tuple(dtype) + (0, 0), base_bytes=tuple(base) + (4, 4)), ["V"])]
    return t, lats, O.solve_config({"target": t, "lattices": lats})


def test_brute_force_matmul_whose_moves_are_specs():
    """The alloc-binding of Section 2 with its load and store Move Specs as children, costed by
    Section 3's equation, against the minimum over all complete programs (the Move Specs'
    programs included, enumerated together with the Matmul's)."""
    t, lats, res = matmul_with_moves([1, 2], levels=2)
    n = brute_force_compare(t, lats, res, "M", pick=lambda s: s.dims[1] * s.dims[2] * s.dims[3] <= 2)
    assert n >= 32
    # with layout and dtype coordinates (three levels): the smallest Specs
    t, lats, res = matmul_with_moves([1, 2], layout=(1, 1, 0), dtype=(1, 0, 0), base=(2, 4, 4))
    n = brute_force_compare(t, lats, res, "M", pick=lambda s: s.dims[1] * s.dims[2] * s.dims[3] == 1)
    assert n >= 200


def test_matmul_with_moves_closed_forms_and_reduction():
    # 1x1x1x1, every operand in memory (level 2), scalar FMA in registers: three loads and one
    # store of one element, each alloc-binding adding a line in memory and a line in the registers
    t, lats, res = matmul_with_moves([1, 2, 4])
    ext = res["M"]["extents"]
    c = res["M"]["cost"].reshape(ext)
    w = t["level_weight"]
    move = 3                       # SCALAR_MOVE
    assert int(c[0, 0, 0, 0, 2, 2, 2]) == 3 * (w[2] + w[0]) + 4 * move + 1
    # a 1x1x4 right-hand side row moved from memory to the vector registers costs two aligned
    # vector moves plus 16 bytes = two lines at either end
    cv = res["V"]["cost"].reshape(res["V"]["extents"])
    assert int(cv[0, 0, 0, 2, 2, 1, 2, 1, 2, 1]) == 2
    # with zero weights and one scalar move microkernel (cost k, no loop constant) every Move Spec of
    # r x c costs r*c*k: the table equals that of the plain Matmul lattice whose Moves cost a
    # coefficient per element (k per load, k per store)
    k = 3
    t = move_target(s=0)
    t["level_weight"] = [0, 0, 0, 0]
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 2), (W.MK_SCALAR_MOVE, 1, k)]
    sizes = [1, 2, 3, 4]
    lats = [("V", move_lattice(sizes, layout=(0, 0), dtype=(0, 0)), []),
            ("M", W._lattice(W.KIND_MATMUL_MOVES, [[1], sizes, sizes, sizes]), ["V"])]
    got = O.solve_config({"target": t, "lattices": lats})["M"]
    for src in range(1, 3):
        for dst in range(src):
            t["load_coef"][src][dst][0] = k
            t["store_coef"][dst][src][0] = k
    plain = O.solve(t, W._lattice(W.KIND_MATMUL_ACCUM, [[1], sizes, sizes, sizes]))
    assert np.array_equal(got["cost"], plain["cost"]) and np.array_equal(got["argmin"], plain["argmin"])
    assert got["n_rewrites"] == plain["n_rewrites"] and got["n_admissible"] == plain["n_admissible"]
    assert (got["cost"] != O.INF).sum() > 100
