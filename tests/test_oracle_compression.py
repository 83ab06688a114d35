"""Pins of the oracle's box merge (Section 4.1, Figure 2): unit rectangles merged with
adjacent equal-valued rectangles whose union fills its bounding box."""
import numpy as np
import pytest

from oracle import brute_force as B
from oracle import oracle as O
from paper_2505_01637_amd import workloads as W

import util


def random_table(ext, n_values, seed, run=3):
    """Blocky random values so that runs exist along every axis."""
    rng = np.random.default_rng(seed)
    coarse = [max(1, (e + run - 1) // run) for e in ext]
    base = rng.integers(0, n_values, size=coarse, dtype=np.uint64)
    idx = np.ix_(*[np.arange(e) // run for e in ext])
    return base[idx].copy()


def check_valid_decomposition(ext, boxes, v0, v1):
    d0, d1, cover = O.decompress(ext, boxes)
    assert (cover == 1).all()                       # disjoint and covering
    assert np.array_equal(d0, v0.ravel()) and np.array_equal(d1, v1.ravel())   # every box constant


def test_merge_matches_dictionary_implementation():
    for seed, ext, mo in [(0, [4, 5, 3], [2, 1, 0]), (1, [3, 4, 2, 2], [1, 0, 3, 2]),
                          (2, [6, 6], [1, 0]), (3, [2, 3, 4, 2, 2], [3, 2, 1, 0, 4])]:
        v0 = random_table(ext, 3, seed, run=2)
        v1 = np.zeros_like(v0)
        want = B.merge_boxes(ext, mo, {x: int(v0[x]) for x in util.all_coords(ext)})
        for by_lines in (False, True):
            got = O.merge(ext, mo, v0.ravel(), v1.ravel(), first_pass_by_lines=by_lines)
            assert [(lo, hi, a) for lo, hi, a, _ in util.boxes_as_tuples(got, len(ext))] == want
            check_valid_decomposition(ext, got, v0, v1)


def test_merge_fixed_point_constant_and_bounds():
    ext, mo = [5, 4, 6], [2, 1, 0]
    v0 = random_table(ext, 4, 5)
    v1 = random_table(ext, 2, 6)
    boxes = O.merge(ext, mo, v0.ravel(), v1.ravel())
    assert 1 <= len(boxes) <= v0.size
    check_valid_decomposition(ext, boxes, v0, v1)
    # merging the decompressed table again gives the same list
    d0, d1, _ = O.decompress(ext, boxes)
    again = O.merge(ext, mo, d0, d1)
    assert boxes.tobytes() == again.tobytes()
    # a constant table is one box spanning the lattice
    one = O.merge(ext, mo, np.full(120, 7, dtype=np.uint64), np.zeros(120, dtype=np.uint64))
    assert len(one) == 1 and list(one[0]["lo"][:3]) == [0, 0, 0] and list(one[0]["hi"][:3]) == [4, 3, 5]
    # all-distinct values cannot merge
    distinct = O.merge(ext, mo, np.arange(120, dtype=np.uint64), np.zeros(120, dtype=np.uint64))
    assert len(distinct) == 120
    # sorted by lo, first axis most significant
    los = [tuple(b["lo"][:3]) for b in boxes]
    assert los == sorted(los)


def test_merge_is_not_a_plain_run_length_encoding():
    """An L-shaped region must split into boxes that each fill their bounding box (Figure 2)."""
    v = np.zeros((3, 3), dtype=np.uint64)
    v[0, :] = 1
    v[:, 0] = 1                      # an L of ones
    boxes = util.boxes_as_tuples(O.merge([3, 3], [1, 0], v.ravel(), np.zeros(9, dtype=np.uint64)), 2)
    assert boxes == [((0, 0), (0, 2), 1, 0), ((1, 0), (2, 0), 1, 0), ((1, 1), (2, 2), 0, 0)]


def test_cost_values_are_reduced_fractions_and_table_roundtrip():
    """Costs are compared after normalising to the Spec's volume (Section 4.1); the
    reduced fraction must reproduce the cost exactly."""
    cfg = W.config(4, seed=4, max_size=16)
    t, lat = cfg["target"], cfg["lattices"][0][1]
    r = O.solve(t, lat)
    ext, mo, _ = O.geometry(t, lat)
    assert mo == [3, 2, 1, 0, 6, 5, 4, 9, 8, 7]
    v0, v1 = O.cost_values(t, lat, r["cost"])
    sizes = [np.array(s, dtype=np.uint64) for s in lat["sizes"]]
    grid = np.indices(ext[:4]).reshape(4, -1)
    vol = np.ones(grid.shape[1], dtype=np.uint64)
    for d in range(4):
        vol *= sizes[d][grid[d]]
    per = int(np.prod(ext[4:]))
    vol = np.repeat(vol, per)
    fin = r["cost"] != O.INF
    assert (v1[~fin] == 0).all() and (v0[~fin] == O.INF).all()
    assert np.array_equal(v0[fin] * (vol[fin] // v1[fin]), r["cost"][fin])
    assert (vol[fin] % v1[fin] == 0).all() and (np.gcd(v0[fin], v1[fin]) == 1).all()
    dec, cst = O.compress_table(t, lat, r["cost"], r["argmin"])
    d0, _, cover = O.decompress(ext, dec)
    assert (cover == 1).all() and np.array_equal(d0.astype(np.uint16), r["argmin"])
    c0, c1, cover = O.decompress(ext, cst)
    assert (cover == 1).all() and np.array_equal(c0, v0) and np.array_equal(c1, v1)
    assert len(dec) < len(r["argmin"]) // 4          # decisions do compress


@pytest.mark.parametrize("number,max_size,label", [(1, None, "M"), (5, 2, "F"), (4, 2, "M")])
def test_point_lookup_in_boxes_equals_dense_table(number, max_size, label):
    """Section 4.1: a lookup in the compressed table returns what the dense table holds.  Pinned
    against the dense fill (itself pinned by brute force): every coordinate of a small table, or a
    seeded sample of a larger one, looked up by scanning the two box lists."""
    cfg = W.config(number, max_size=max_size)
    res = O.solve_config(cfg)
    lat = next(l for lb, l, _ in cfg["lattices"] if lb == label)
    r = res[label]
    ext = r["extents"]
    dec, cst = O.compress_table(cfg["target"], lat, r["cost"], r["argmin"])
    n = len(r["cost"])
    pick = np.arange(n) if n <= 3000 else np.random.default_rng(7).choice(n, size=3000, replace=False)
    coords = np.stack(np.unravel_index(pick, ext), axis=1)
    cost, arg = O.query_boxes(lat, dec, cst, coords)
    assert np.array_equal(cost, r["cost"][pick]) and np.array_equal(arg, r["argmin"][pick])
    assert (cost != np.uint64(O.INF)).any()
    # a planted mistake is seen: one box moved by one cell no longer partitions the lattice
    broken = dec.copy()
    i = int(np.argmax(broken["hi"][:, 3] - broken["lo"][:, 3]))
    if broken["hi"][i, 3] > broken["lo"][i, 3]:
        broken["hi"][i, 3] -= 1
        with pytest.raises(ValueError):
            O.query_boxes(lat, broken, cst, np.stack(np.unravel_index(np.arange(n), ext), axis=1)[: 20000])


@pytest.mark.parametrize("number,max_size", [(4, 8), (3, 64), (5, 4)])
def test_first_pass_by_lines_equals_the_unit_box_pass_on_solved_tables(number, max_size):
    """orc_merge's default first pass walks the lines of the first merge axis instead of sorting
    one unit box per cell.  On the lists that matter, the decisions and the volume-normalised
    costs (reduced fractions, v1 != 0) of solved tables, both forms must give the same boxes."""
    cfg = W.config(number, max_size=max_size)
    res = O.solve_config(cfg)
    for label, lat, _ in cfg["lattices"]:
        ext, mo, _ = O.geometry(cfg["target"], lat)
        v0, v1 = O.cost_values(cfg["target"], lat, res[label]["cost"])
        assert (v1 != 0).any() and len(np.unique(v1)) > 2
        for a0, a1 in ((v0, v1), (res[label]["argmin"].astype(np.uint64), np.zeros(len(v0), dtype=np.uint64))):
            by_lines = O.merge(ext, mo, a0, a1, first_pass_by_lines=True)
            by_cells = O.merge(ext, mo, a0, a1, first_pass_by_lines=False)
            assert by_lines.tobytes() == by_cells.tobytes()
            assert len(by_lines) < len(a0)
