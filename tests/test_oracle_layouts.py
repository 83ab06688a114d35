"""Pins of the packed and the shuffled layout (Section 2.4.2) and of what they do to a tile's
contiguousness and alignment (Section 2.4.3) in the oracle's Move lattice and in the Matmul
lattice whose Moves are Move Specs."""
import itertools

import numpy as np
import pytest

from oracle import brute_force as B
from oracle import oracle as O
from paper_2505_01637_amd import workloads as W

import util
from test_oracle_pins import brute_force_compare
from test_oracle_moves import move_target


def test_layout_offsets_are_the_printed_expressions():
    # the odd-even shuffle of Section 2.4.2, sigma(s, x) = 2 (x mod s/2) + floor(2x / s), for s = 8:
    # the first half of a strip goes to the even places, the second half to the odd ones
    assert [O.layout_offset(3, 1, 8, 8, 0, j) for j in range(8)] == [0, 2, 4, 6, 1, 3, 5, 7]
    assert [O.layout_offset(3, 1, 4, 4, 0, j) for j in range(4)] == [0, 2, 1, 3]
    # 2 x 4 in strips of 2: strip 0 holds columns 0, 1 of both rows, then strip 1
    got = [[O.layout_offset(2, 2, 4, 2, i, j) for j in range(4)] for i in range(2)]
    assert got == [[0, 1, 4, 5], [2, 3, 6, 7]]
    assert [[O.layout_offset(0, 2, 3, 2, i, j) for j in range(3)] for i in range(2)] == [[0, 1, 2], [3, 4, 5]]
    assert [[O.layout_offset(1, 2, 3, 2, i, j) for j in range(3)] for i in range(2)] == [[0, 2, 4], [1, 3, 5]]
    # one row in whole strips is the same sequence of values as a row-major row
    assert [O.layout_offset(2, 1, 12, 4, 0, j) for j in range(12)] == list(range(12))


@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_layout_offsets_are_bijections(layout):
    for rows, cols, s in [(1, 4, 2), (3, 8, 4), (5, 12, 2), (4, 16, 8), (7, 6, 6)]:
        offs = sorted(O.layout_offset(layout, rows, cols, s, i, j) for i in range(rows) for j in range(cols))
        assert offs == list(range(rows * cols)), (layout, rows, cols, s)


def groups_are_ranges(offsets_by_group):
    return all(sorted(g) == list(range(min(g), min(g) + len(g))) for g in offsets_by_group)


@pytest.mark.parametrize("layout", [0, 1, 2, 3])
def test_tile_transfer_functions_are_sound_for_the_layout(layout):
    """What the transfer functions of Section 2.4.3 claim about a tile of a fresh tensor must hold
    for the buffer offsets of the layout, at every position of the tile: with k inner physical
    dimensions adjacent, the tile's values that share the outer coordinates fill a range of
    offsets without holes; an aligned tile starts at a multiple of the cache line."""
    strip, line = 4, 16
    t = move_target(line_bytes=line)
    t["strip"] = strip
    for rows, cols in [(4, 8), (2, 16), (8, 4), (1, 8), (6, 12)]:
        if layout >= 2 and cols % strip:
            continue
        nd = 3 if layout >= 2 else 2
        ly = (layout, layout)
        spec = B.Spec(B.V, (1, rows, 1, cols), (2, 1), ly, (0, 0), (), (nd, nd), (1, 1))
        for r2, c2 in itertools.product([d for d in range(1, rows + 1) if rows % d == 0], [d for d in range(1, cols + 1) if cols % d == 0]):
            if layout >= 2 and c2 % strip and strip % c2:
                continue
            contig, aligned = B.tiled_tensor(t, spec, 0, r2, c2)
            assert (0 if layout == 3 else 1) <= contig <= nd
            for i0, j0 in itertools.product(range(0, rows, r2), range(0, cols, c2)):
                cells = [(i, j) for i in range(i0, i0 + r2) for j in range(j0, j0 + c2)]
                off = {c: O.layout_offset(layout, rows, cols, strip, *c) for c in cells}
                # outer physical coordinates of a cell: what is left after dropping the `contig` inner dimensions
                def outer(c):
                    i, j = c
                    phys = (i, j) if layout == 0 else (j, i) if layout == 1 else (j // strip, i, j % strip)
                    return phys[:nd - contig]
                groups = {}
                for c in cells:
                    groups.setdefault(outer(c), []).append(off[c])
                assert groups_are_ranges(groups.values()), (layout, rows, cols, r2, c2, contig)
                if aligned:
                    assert (min(off.values()) * 4) % line == 0, (layout, rows, cols, r2, c2)
    # and the claims are not vacuous: a whole strip of a packed tensor is contiguous, a block of the
    # same shape cut out of a row-major tensor is not
    packed = B.Spec(B.V, (1, 4, 1, 8), (2, 1), (2, 2), (0, 0), (), (3, 3), (1, 1))
    plain = B.Spec(B.V, (1, 4, 1, 8), (2, 1), (0, 0), (0, 0), (), (2, 2), (1, 1))
    assert B.tiled_tensor(t, packed, 0, 4, 4) == (3, 1)
    assert B.tiled_tensor(t, plain, 0, 4, 4) == (1, 1)
    # a tile narrower than a strip: the same two columns of every row of one strip; in a shuffled
    # strip those two columns are not neighbours
    assert B.tiled_tensor(t, packed, 0, 4, 2) == (1, 0)
    assert B.tiled_tensor(t, packed._replace(layouts=(3, 3)), 0, 4, 2) == (0, 0)
    assert B.tiled_tensor(t, packed._replace(layouts=(3, 3)), 0, 4, 1) == (1, 0)


def packed_move_lattice(sizes, layout=(2, 2), dtype=(0, 0)):
    return W._lattice(W.KIND_MOVE, [[1], list(sizes), [1], list(sizes)], layout=layout + (0, 0, 0), dtype=dtype + (0, 0, 0))


def test_brute_force_move_lattice_with_packed_layouts():
    """Every Spec of a Move lattice over sizes {1, 2, 4} with all four layouts on both tensors,
    strips of two columns, three levels, against the minimum over all complete programs."""
    t = move_target(line_bytes=8)
    t["strip"] = 2
    lats = [("V", packed_move_lattice([1, 2, 4]), [])]
    res = O.solve_config({"target": t, "lattices": lats})
    assert res["V"]["extents"] == [1, 3, 1, 3, 3, 3, 4, 2, 4, 2, 4, 4]
    n = brute_force_compare(t, lats, res, "V")
    assert n == len(res["V"]["cost"]) == 9 * 9 * 64 * 16
    ext = res["V"]["extents"]
    c = res["V"]["cost"].reshape(ext)
    # one column of a strip of two has at most that column adjacent; a row-major tensor has no three adjacent dimensions
    assert (c[0, :, 0, 0, :, :, 2:, :, :, :, 2:, :] == O.INF).all() and (c[0, :, 0, 0, :, :, :, :, 2:, :, :, 2:] == O.INF).all()
    assert (c[0, :, 0, :, :, :, 3, :, :, :, :2, :] == O.INF).all()
    assert (c[0, :, 0, 0, :, :, :2, :, :2, :, 2:, 2:] != O.INF).all()
    assert res["V"]["n_admissible"] == int((c != O.INF).sum()) < len(res["V"]["cost"])


def test_packed_layout_closed_forms():
    """Strips of 4 columns, cache lines of 16 bytes (4 f32), 4-lane vector moves (aligned ones cost
    1, plain ones 2, scalar moves 3), no loop constant.  Moving a 4 x 8 tensor from memory (level 2)
    into vector registers (level 1):"""
    t = move_target(line_bytes=16, s=0, lanes=4)
    t["strip"] = 4
    lat = packed_move_lattice([1, 2, 4, 8])
    ext = W.coord_extents(t, lat)
    r = O.solve(t, lat)
    c = r["cost"].reshape(ext)
    i = {1: 0, 2: 1, 4: 2, 8: 3}
    at = lambda rows, cols, cs, as_, cd, ad, ys, yd: int(c[0, i[rows], 0, i[cols], 2, 1, cs, as_, cd, ad, ys, yd])
    # row-major to row-major, both fresh: rows of 32 bytes are whole lines: 8 aligned vector moves
    assert at(4, 8, 2, 1, 2, 1, 0, 0) == 8
    # packed to packed, both fresh: the same
    assert at(4, 8, 3, 1, 3, 1, 2, 2) == 8
    # shuffled to shuffled likewise; shuffled to plain packed has no vector move (the vectors hold other values): 32 scalar moves
    assert at(4, 8, 3, 1, 3, 1, 3, 3) == 8
    assert at(4, 8, 3, 1, 3, 1, 3, 2) == 32 * 3
    # half a strip of a packed row (2 of 4 columns, 4-lane vectors): element by element
    assert at(1, 2, 1, 0, 1, 0, 2, 2) == 2 * 3
    # row-major to packed: a row of the row-major tensor and a row of a strip are both whole lines here
    assert at(4, 8, 2, 1, 3, 1, 0, 2) == 8
    # a 4 x 4 tile: rows of 16 bytes; cut out of the fresh row-major 4 x 8 tensor it is aligned still
    # (every suffix a whole line), and so is a whole strip of the packed one
    # bf16 makes the difference: rows of a 4 x 8 bf16 row-major tensor are 16 bytes, of its 4 x 4 tiles 8
    lat16 = packed_move_lattice([1, 2, 4, 8], dtype=(1, 1))
    ext16 = W.coord_extents(t, lat16)
    c16 = O.solve(t, lat16)["cost"].reshape(ext16)
    at16 = lambda rows, cols, cs, as_, cd, ad, ys, yd: int(c16[0, i[rows], 0, i[cols], 2, 1, cs, as_, cd, ad, ys, yd, 1, 1])
    # one row of 8 bf16 = one line, fresh, row-major both sides: two aligned 4-lane moves
    assert at16(1, 8, 2, 1, 2, 1, 0, 0) == 2
    # 4 x 8 bf16 row-major: tiles of one row are whole lines: 4 rows x 2 aligned moves
    assert at16(4, 8, 2, 1, 2, 1, 0, 0) == 8
    # 4 x 8 bf16 packed in strips of 4: a row of a strip is 8 bytes, half a line: its one-row tiles
    # are not known to be aligned, so the plain vector move (2) does them: 8 rows of strips x 2
    assert at16(4, 8, 3, 1, 3, 1, 2, 2) == 16
    # monotone in what is known, with the packed layouts too
    for axis in (6, 7, 8, 9):
        x = np.moveaxis(c, axis, 0)
        fin = (x[1:] != O.INF) & (x[:-1] != O.INF)
        assert (x[1:][fin] <= x[:-1][fin]).all()


def matmul_with_packed_moves(sizes, layout=(1, 2, 2), levels=3, strip=2, lanes=2):
    t = move_target(lanes=lanes)
    t["strip"] = strip
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 1), (W.MK_BCAST_VEC_MULADD, lanes, 1)] + t["microkernels"]
    if levels == 2:
        t["n_levels"] = 2
        t["capacity_bytes"] = [64, W.UNBOUNDED, 0, 0]
    lats = [("V", packed_move_lattice(sizes), []),
            ("M", W._lattice(W.KIND_MATMUL_MOVES, [[1], list(sizes), list(sizes), list(sizes)], layout=tuple(layout) + (0, 0)), ["V"])]
    return t, lats, O.solve_config({"target": t, "lattices": lats})


def test_brute_force_matmul_with_packed_operands():
    t, lats, res = matmul_with_packed_moves([1, 2], levels=2)
    assert res["M"]["extents"] == [1, 2, 2, 2, 2, 2, 2, 2, 4, 4]
    n = brute_force_compare(t, lats, res, "M", pick=lambda s: s.dims[1] * s.dims[2] * s.dims[3] <= 2)
    assert n >= 300
    t, lats, res = matmul_with_packed_moves([1, 2])
    n = brute_force_compare(t, lats, res, "M", pick=lambda s: s.dims[1] * s.dims[2] * s.dims[3] == 1 or
                            (s.dims == (1, 1, 1, 2) and sum(s.levels[:3]) <= 3))
    assert n >= 400
    # an operand packed in less than a strip does not exist (operands are whole tensors); the vector microkernel takes a packed row
    c = res["M"]["cost"].reshape(res["M"]["extents"])
    assert (c[0, :, :, 0, :, :, :, :, 2:, :] == O.INF).all() and (c[0, :, :, 0, :, :, :, :, :, 2:] == O.INF).all()
    ids = O.geometry(t, lats[1][1])[2]
    a = res["M"]["argmin"].reshape(res["M"]["extents"])
    assert int(a[0, 0, 0, 1, 0, 1, 1, 0, 2, 2]) == 1 and int(a[0, 0, 0, 1, 0, 1, 1, 0, 0, 2]) == 1     # select(BroadcastVecMultAdd)
    assert int(a[0, 0, 0, 1, 0, 1, 1, 0, 3, 0]) != 1                                                    # not on shuffled strips
    assert ids["tile_base"] == ids["move_base"] + 3 * 2 * 8


def test_matmul_lattice_rejects_a_move_table_without_the_packed_layouts():
    t = move_target()
    t["strip"] = 2
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 1)] + t["microkernels"]
    v = W._lattice(W.KIND_MOVE, [[1], [1, 2], [1], [1, 2]], layout=(1, 1, 0, 0, 0))
    m = W._lattice(W.KIND_MATMUL_MOVES, [[1], [1, 2], [1, 2], [1, 2]], layout=(0, 2, 0, 0, 0))
    rv = O.solve(t, v)
    with pytest.raises(ValueError):
        O.solve(t, m, deps=((v, rv["cost"]),))
    # packed layouts only where Moves are Specs
    with pytest.raises(ValueError):
        O.solve(t, W._lattice(W.KIND_MATMUL_ACCUM, [[1], [1, 2], [1, 2], [1, 2]], layout=(0, 2, 0, 0, 0)))
    t["strip"] = 3
    with pytest.raises(ValueError):
        O.solve(t, W._lattice(W.KIND_MOVE, [[1], [1, 2], [1], [1, 2]], layout=(2, 2, 0, 0, 0)))
