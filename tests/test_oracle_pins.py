"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU or the HIP library.
"""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import brute_force as B
from oracle import oracle as O
from paper_2505_01637_amd import workloads as W

import util

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
UNB = W.UNBOUNDED


def fig1_setup():
    g = json.load(open(os.path.join(GOLDEN, "fig1_worked_example.json")))
    t = W._empty_target(4, g["capacity_bytes"])
    idx = {"RF": 0, "VRF": 1, "L1": 2, "GL": 3}
    for pair, coef in g["move_coef_by_level_pair"].items():
        src, dst = (idx[p] for p in pair.split("-"))
        t["load_coef"][src][dst][0] = coef
        t["store_coef"][dst][src][0] = coef
    t["loop_overhead"] = g["loop_overhead"]
    t["microkernels"] = [tuple(m) for m in g["microkernels"]]
    s = g["sizes"]
    lat = W._lattice(W.KIND_MATMUL_ACCUM, [s["b"], s["m"], s["k"], s["n"]])
    return g, t, lat


def test_fig1_steps_are_rewrites_and_cost_matches_hand_derivation():
    """Figure 1 / Section 2: every step of the example lowering is an applicable
    rewrite, and Section 3's equation gives the hand-derived cost."""
    g, t, lat = fig1_setup()
    lats = {0: lat}
    goal = B.Spec(0, (1, 4, 4, 16), (0, 1, 2, 0, 0), (0,) * 5, (0,) * 5)
    # tile([1,1,1,16]) as tile m -> 1 then tile k -> 1 (Section 4: single-dimension tiles)
    step = {rid: (node, ch) for rid, node, ch in B.rewrites(t, lats, goal)}
    tile_m = [(rid, v) for rid, v in step.items() if v[0][0] == "loop" and v[1][0].dims == (1, 1, 4, 16)]
    assert len(tile_m) == 1 and tile_m[0][1][0][1] == 4
    s1 = tile_m[0][1][1][0]
    step = {rid: (node, ch) for rid, node, ch in B.rewrites(t, lats, s1)}
    tile_k = [v for v in step.values() if v[0][0] == "loop" and v[1][0].dims == (1, 1, 1, 16)]
    assert len(tile_k) == 1 and tile_k[0][0][1] == 4
    s2 = tile_k[0][1][0]
    assert s2.levels[:3] == (0, 1, 2)
    # move_param(2, VRF): output L1 -> VRF pays a load and a store
    moves = [(node, ch) for rid, node, ch in B.rewrites(t, lats, s2)
             if node[0] == "alloc" and ch[0].levels[:3] == (0, 1, 1)]
    assert len(moves) == 1 and moves[0][0][1] == (2 + 2) * 16
    s3 = moves[0][1][0]
    # select(BroadcastVecMultAdd)
    leaves = [node for rid, node, ch in B.rewrites(t, lats, s3) if node[0] == "mk"]
    assert leaves == [("mk", 2)]
    leaf = ("mk", 2)
    alloc = ("alloc", 64, leaf)
    kloop = ("loop", 4, 1, alloc)
    mloop = ("loop", 4, 1, kloop)
    d = list(g["hand_derivation"].values())
    assert [B.c(leaf), B.c(alloc), B.c(kloop), B.c(mloop)] == d
    assert B.c(mloop) == g["figure1_schedule_cost"] == 1061


def test_fig1_dp_optimum():
    """The oracle's optimum for the Figure 1 goal equals the hand-derived 293 and
    does not exceed the example schedule's 1061; ties go to the lowest id."""
    g, t, lat = fig1_setup()
    r = O.solve(t, lat)
    ext, _, ids = O.geometry(t, lat)
    goal = B.Spec(0, (1, 4, 4, 16), (0, 1, 2, 0, 0), (0,) * 5, (0,) * 5)
    x = util.linear(ext, util.coord_of_spec(t, lat, goal))
    assert int(r["cost"][x]) == g["optimum_cost"] == 293
    assert int(r["cost"][x]) <= g["figure1_schedule_cost"]
    # move operand 2 to level 1, same layout, no convert
    assert int(r["argmin"][x]) == ids["move_base"] + ((2 * 3 + 1) * 2 + 0) * 2 + 0
    # the sub-spec 1x1x1x16 RF,VRF,L1 on its own: brute force over every schedule
    sub = B.Spec(0, (1, 1, 1, 16), (0, 1, 2, 0, 0), (0,) * 5, (0,) * 5)
    best, arg, cnt = B.optimum(t, {0: lat}, sub)
    xs = util.linear(ext, util.coord_of_spec(t, lat, sub))
    assert cnt > 1 and best == int(r["cost"][xs]) and arg == int(r["argmin"][xs])


def brute_force_compare(target, lattices, results, label, pick=lambda spec: True, cap=None):
    lat = next(l for lb, l, _ in lattices if lb == label)
    lats = {l["kind"]: l for _, l, _ in lattices}
    ext = W.coord_extents(target, lat)
    res = results[label]
    checked = 0
    n_rw = 0
    for x in util.all_coords(ext):
        spec = util.spec_of_coord(target, lat, x)
        n_rw += B.count_rewrites(target, lats, spec)
        if not pick(spec):
            continue
        best, arg, cnt = B.optimum(target, lats, spec)
        i = util.linear(ext, x)
        if best is None:
            assert int(res["cost"][i]) == O.INF and int(res["argmin"][i]) == O.NONE, (spec,)
        else:
            assert int(res["cost"][i]) == best, (spec, best)
            assert int(res["argmin"][i]) == arg, (spec, arg)
        checked += 1
    assert n_rw == res["n_rewrites"]
    return checked


def test_brute_force_two_levels():
    """Optimal substructure (Section 3): the memoized search equals the minimum of
    c(p) over every complete schedule; all specs of a 2-level lattice with sizes {1,2,3,4}."""
    cfg = W.config(1, seed=11, max_size=4)
    cfg["target"]["loop_overhead"] = 2
    res = O.solve_config(cfg)
    big = lambda s: s.dims[1] * s.dims[2] * s.dims[3] <= 32
    n = brute_force_compare(cfg["target"], cfg["lattices"], res, "M", pick=big)
    assert n >= 400


def small_four_level(seed, transposed=False):
    rng = W.SplitMix64(seed)
    t, w = W._four_level_target(rng)
    if transposed:
        W._add_transposed(t, rng)
    return t, w


def test_brute_force_four_levels_vector_microkernel():
    """Same check with RF/VRF/L1/GL, BroadcastVecMultAdd and capacities that bite."""
    t, _ = small_four_level(5)
    lat = W._lattice(W.KIND_MATMUL_ACCUM, [[1], [1, 2], [1, 2], [1, 8, 16]])
    res = {"M": O.solve(t, lat)}
    pick = lambda s: sum(s.levels[:3]) <= 4
    n = brute_force_compare(t, [("M", lat, [])], res, "M", pick=pick)
    assert n > 200


def test_brute_force_layout_and_dtype_coordinates():
    """bf16 inputs with convert-Moves, a transposing Move and the bf16 dot kernel."""
    cfg = W.config(3, seed=7)
    t = cfg["target"]
    lat = W._lattice(W.KIND_MATMUL_ACCUM, [[1], [1], [1, 16, 32], [1, 2, 8]],
                     layout=(0, 1, 0, 0, 0), dtype=(1, 1, 0, 0, 0), base_bytes=(2, 2, 4, 4, 4))
    res = {"M": O.solve(t, lat)}
    pick = lambda s: sum(s.levels[:3]) <= 3
    n = brute_force_compare(t, [("M", lat, [])], res, "M", pick=pick)
    assert n > 300
    # a bf16 operand already in RF can no longer be converted: such specs have no program
    c = res["M"]["cost"]
    assert (c == O.INF).sum() > 0


def test_brute_force_fused_pipeline():
    """Kind E and kind F (bufferize = pipeline node costing the sum of its children,
    Section 3) on a tiny lattice; this build's own reading of Section 2.1."""
    cfg = W.config(5, seed=3)
    t = cfg["target"]
    r = [1, 2]
    n8 = [1, 8]
    lats = [("M", W._lattice(W.KIND_MATMUL_ACCUM, [[1], r, r, n8], layout=(1, 1, 1, 0, 0)), []),
            ("E", W._lattice(W.KIND_BIAS_ADD_RELU, [[1], r, [1], n8], layout=(1, 0, 1, 0, 0)), []),
            ("F", W._lattice(W.KIND_FUSED_MM_ADD_RELU, [[1], r, r, n8], layout=(1, 1, 0, 1, 0)), ["M", "E"])]
    res = O.solve_config({"target": t, "lattices": lats})
    n = brute_force_compare(t, lats, res, "E", pick=lambda s: sum(s.levels[:3]) <= 4)
    assert n > 100
    n = brute_force_compare(t, lats, res, "F",
                            pick=lambda s: sum(s.levels[:4]) + s.levels[4] <= 2 and s.dims[1] * s.dims[3] <= 8)
    assert n > 100
    # the fused lattice may distinguish a tensor's layout only if the table it is looked up in does
    import pytest
    lats[1] = ("E", dict(lats[1][1], layout_coord=[1, 0, 0, 0, 0]), [])
    with pytest.raises(ValueError):
        O.solve_config({"target": t, "lattices": lats})


def parallel_setup(threads, sync, max_size=4):
    cfg = W.config(1, seed=11, max_size=max_size)
    t = cfg["target"]
    t["loop_overhead"] = 2
    t["threads"], t["sync_cost"] = threads, sync
    lat_m = cfg["lattices"][0][1]
    lat_p = dict(lat_m, kind=W.KIND_MATMUL_PARALLEL)
    lats = [("M", lat_m, []), ("P", lat_p, ["M"])]
    return t, lats, O.solve_config({"target": t, "lattices": lats})


def test_brute_force_parallel_loops():
    """Section 3's loop rule with threads > 1: ceil(trips / threads) * c(body) + s, the body being
    serial-only (Section 2.2).  Three threads over sizes {1,2,3,4} exercise the rounding up (4
    trips = 2 rounds, 2 and 3 trips = 1 round); every Spec up to volume 32 against the minimum
    over all complete programs."""
    t, lats, res = parallel_setup(threads=3, sync=7)
    big = lambda s: s.dims[1] * s.dims[2] * s.dims[3] <= 32
    n = brute_force_compare(t, lats, res, "P", pick=big)
    assert n >= 400
    cm, cp = res["M"]["cost"], res["P"]["cost"]
    assert (cp <= cm).all() and (cp < cm).any()
    assert ((cp == O.INF) == (cm == O.INF)).all()
    _, _, ids = O.geometry(t, lats[1][1])
    assert (res["P"]["argmin"][cp < cm] != res["M"]["argmin"][cp < cm]).any()
    assert (res["P"]["argmin"][cp != O.INF] > ids["bufferize"]).any()        # parallel-loop ids are in use
    # a closed form: 1x4x1x1 with everything in RF is 4 scalar FMAs; serial = 4*1 + 2, three
    # threads = 2 rounds * 1 + 7: the serial loop stays; with 4 threads and s = 3: 1 + 3 wins
    ext = res["P"]["extents"]
    x = util.linear(ext, (0, 3, 0, 0, 0, 0, 0))
    mk = t["microkernels"][0][2]
    assert int(cm[x]) == 4 * mk + 2 and int(cp[x]) == min(4 * mk + 2, 2 * mk + 7)
    t4, lats4, res4 = parallel_setup(threads=4, sync=3)
    assert int(res4["P"]["cost"][x]) == mk + 3
    assert int(res4["P"]["argmin"][x]) == ids["bufferize"] + 1 + 1 * ids["maxs"] + 0


def test_parallel_table_with_one_thread_is_the_serial_table():
    """threads = 1 and s equal to the loop constant make a parallel loop cost exactly what the
    serial loop costs; ties go to the lower (serial) id, so both tables agree entry by entry."""
    t, lats, res = parallel_setup(threads=1, sync=2, max_size=6)
    assert np.array_equal(res["P"]["cost"], res["M"]["cost"])
    assert np.array_equal(res["P"]["argmin"], res["M"]["argmin"])
    assert res["P"]["n_rewrites"] > res["M"]["n_rewrites"]


def bounded_setup(caps=(16, 64), sizes=(1, 2, 4)):
    """Two levels, both of finite capacity: bounds 0,1,..,16 B on level 0 and 0,1,..,64 B on level 1."""
    cfg = W.config(1, seed=11, max_size=4)
    t = cfg["target"]
    t["loop_overhead"] = 2
    t["capacity_bytes"][0], t["capacity_bytes"][1] = caps
    r = list(sizes)
    lat = W._lattice(W.KIND_MATMUL_BOUNDED, [[1], r, r, r])
    lats = [("B", lat, [])]
    return t, lats, O.solve_config({"target": t, "lattices": lats})


def test_brute_force_memory_bounds():
    """Sections 2.2 and 2.4.4: the per-level memory bounds are coordinates; a Move takes the moved
    buffer's bytes out of the destination level's bound and the rest is rounded down to a power
    of two.  Every Spec of a small lattice against the minimum over all complete programs."""
    t, lats, res = bounded_setup()
    ext = res["B"]["extents"]
    assert ext == [1, 3, 3, 3, 2, 2, 2, 6, 8]
    n = brute_force_compare(t, lats, res, "B", pick=lambda s: s.dims[1] * s.dims[2] * s.dims[3] <= 16)
    assert n > 5000
    # more memory never hurts: the cost does not rise along either bound axis
    c = res["B"]["cost"].reshape(ext)
    for axis in (7, 8):
        a = np.moveaxis(c, axis, 0)
        assert (a[1:] <= a[:-1]).all()
    assert (c[..., 0, :] > c[..., 5, :]).any()
    # closed form: 1x1x1x1 with every operand in level 1 needs three 4-byte buffers in level 0
    # for the scalar FMA.  Bound 16: 16 -> 12 -> 8, 8 -> 4, 4 -> 0: it fits.  Bound 8: 8 -> 4,
    # 4 -> 0, and the third Move finds nothing left, although 12 bytes would have done without
    # the rounding.
    ld, st = t["load_coef"][1][0][0], t["store_coef"][0][1][0]
    mk = t["microkernels"][0][2]
    assert int(c[0, 0, 0, 0, 1, 1, 1, 5, 0]) == 3 * ld + st + mk
    assert int(c[0, 0, 0, 0, 1, 1, 1, 4, 7]) == O.INF
    assert int(c[0, 0, 0, 0, 0, 0, 0, 0, 0]) == mk          # nothing to allocate: bounds of zero do
    # a Spec that is already in level 0 but larger than one element tiles down without memory
    assert int(c[0, 1, 0, 0, 0, 0, 0, 0, 0]) == 2 * mk + 2


def bounded_fused_setup(caps=(16, 64)):
    """Two levels of finite capacity; Matmul, bias-add + ReLU and fused tables, all with bounds."""
    t = W._empty_target(2, caps)
    t["load_coef"][1][0][0], t["store_coef"][0][1][0] = 3, 5
    t["loop_overhead"] = 1
    t["zero_coef"] = [1, 2, 0, 0]
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 2), (W.MK_SCALAR_ADDRELU, 1, 1), (W.MK_VEC_ADDRELU, 2, 1)]
    r = [1, 2]
    lats = [("M", W._lattice(W.KIND_MATMUL_BOUNDED, [[1], r, r, r]), []),
            ("E", W._lattice(W.KIND_BIAS_ADD_RELU_BOUNDED, [[1], r, [1], r]), []),
            ("F", W._lattice(W.KIND_FUSED_BOUNDED, [[1], r, r, r]), ["M", "E"])]
    return t, lats, O.solve_config({"target": t, "lattices": lats})


def test_brute_force_memory_bounds_through_a_pipeline():
    """Section 2.4.4, second case: a pipeline allocates its intermediate, so both of its stages
    get the intermediate's level's bound lowered by its bytes and snapped down.  The bounded
    bias-add + ReLU table and the bounded fused table against all complete programs."""
    t, lats, res = bounded_fused_setup()
    n = brute_force_compare(t, lats, res, "E")
    assert n == len(res["E"]["cost"])
    n = brute_force_compare(t, lats, res, "F", pick=lambda s: s.dims[1] * s.dims[2] * s.dims[3] <= 4)
    assert n > 3000
    ext = res["F"]["extents"]
    assert ext == [1, 2, 2, 2, 2, 2, 2, 2, 2, 6, 8]
    c = res["F"]["cost"].reshape(ext)
    for axis in (9, 10):                                  # more memory never hurts
        a = np.moveaxis(c, axis, 0)
        assert (a[1:] <= a[:-1]).all()
    # closed form: 1x1x1x1, everything in level 0, intermediate in level 0: the pipeline needs the
    # intermediate's 4 bytes of level 0's bound: zero[0]*1 + FMA + add+ReLU with a bound of 4, nothing with 2
    assert int(c[0, 0, 0, 0, 0, 0, 0, 0, 0, 3, 0]) == 1 + 2 + 1
    assert int(c[0, 0, 0, 0, 0, 0, 0, 0, 0, 2, 7]) == O.INF
    _, _, ids = O.geometry(t, lats[2][1])
    assert int(res["F"]["argmin"].reshape(ext)[0, 0, 0, 0, 0, 0, 0, 0, 0, 3, 0]) == ids["bufferize"]


def test_memory_bounds_that_never_bind_give_the_unbounded_table():
    """With bounds far above every allocation the bounded table at its top bounds is the plain
    Matmul table of a target whose levels are unbounded (pinned above by brute force)."""
    t, lats, res = bounded_setup(caps=(1 << 20, 1 << 20), sizes=(1, 2, 3, 4))
    ext = res["B"]["extents"]
    top = res["B"]["cost"].reshape(ext)[..., ext[7] - 1, ext[8] - 1]
    top_arg = res["B"]["argmin"].reshape(ext)[..., ext[7] - 1, ext[8] - 1]
    t2 = dict(t, capacity_bytes=[W.UNBOUNDED, W.UNBOUNDED, 0, 0])
    plain = O.solve(t2, dict(lats[0][1], kind=W.KIND_MATMUL_ACCUM))
    assert np.array_equal(top.ravel(), plain["cost"]) and np.array_equal(top_arg.ravel(), plain["argmin"])


def test_closed_forms():
    """Special cases that reduce to closed forms."""
    # (i) scalar FMA only, s = 0: an all-RF spec costs m*k*n*k_fma whenever it fits
    cfg = W.config(1, seed=2)
    t, lat = cfg["target"], cfg["lattices"][0][1]
    t["loop_overhead"] = 0
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 3)]
    r = O.solve(t, lat)
    ext = r["extents"]
    c = r["cost"].reshape(ext)
    for m, k, n in itertools.product(range(1, 17), repeat=3):
        fits = 4 * (m * k + k * n + m * n) <= 256
        v = int(c[0, m - 1, k - 1, n - 1, 0, 0, 0])
        assert v == (3 * m * k * n if fits else O.INF)
    # (ii) prime extent p, others 1, all RF: the only rewrite is tile -> 1, so C = p*k + s
    t["loop_overhead"] = 4
    r = O.solve(t, lat)
    c = r["cost"].reshape(ext)
    a = r["argmin"].reshape(ext)
    _, _, ids = O.geometry(t, lat)
    for p in (2, 3, 5, 7, 11, 13):
        assert int(c[0, p - 1, 0, 0, 0, 0, 0]) == 3 * p + 4
        assert int(c[0, 0, 0, p - 1, 0, 0, 0]) == 3 * p + 4
        assert int(a[0, 0, p - 1, 0, 0, 0, 0]) == ids["tile_base"] + 2 * ids["maxs"] + 0
    # (iii) 1x1x1x1 with everything in L1: loads of all three + store of the output + FMA
    ld, st = t["load_coef"][1][0][0], t["store_coef"][0][1][0]
    assert int(c[0, 0, 0, 0, 1, 1, 1]) == 3 * ld + st + 3
    # lowest id wins the tie between the three Move orders: operand 0 first
    assert int(a[0, 0, 0, 0, 1, 1, 1]) == ids["move_base"] + 0


def test_invariants_and_fill_order_independence():
    """Section 3: a node costs no less than its sub-nodes; Section 2.4.1: a Spec's
    optimum depends only on the Spec, so the order in which goals are solved is irrelevant."""
    cfg = W.config(4, seed=9, max_size=8)
    t, lat = cfg["target"], cfg["lattices"][0][1]
    r0 = O.solve(t, lat)
    n = len(r0["cost"])
    rng = np.random.default_rng(0)
    for goals in (rng.permutation(n), np.arange(n)[::-1].copy()):
        r1 = O.solve(t, lat, goals=goals.astype(np.uint64))
        assert np.array_equal(r0["cost"], r1["cost"]) and np.array_equal(r0["argmin"], r1["argmin"])
        assert r0["n_rewrites"] == r1["n_rewrites"] and r0["n_admissible"] == r1["n_admissible"]
    assert np.array_equal(r0["cost"] == O.INF, r0["argmin"] == O.NONE)
    # every admissible spec of this lattice is solvable (tile to 1, then move everything to RF)
    assert (r0["cost"] != O.INF).sum() == r0["n_admissible"]
    # monotone along the chosen rewrite: C[S] >= C[sub] for tiles and moves
    ext, _, ids = O.geometry(t, lat)
    lats = {0: lat}
    checked = 0
    for i in rng.choice(n, size=3000, replace=False):
        if r0["cost"][i] == O.INF:
            continue
        x = np.unravel_index(i, ext)
        spec = util.spec_of_coord(t, lat, x)
        for rid, node, ch in B.rewrites(t, lats, spec):
            if rid == int(r0["argmin"][i]) and ch:
                j = util.linear(ext, util.coord_of_spec(t, lat, ch[0]))
                assert r0["cost"][j] != O.INF and r0["cost"][i] >= r0["cost"][j]
                # and the stored cost is exactly the affine function of the sub-cost
                sub = ("mk", int(r0["cost"][j]))
                assert B.c(node + (sub,)) == int(r0["cost"][i])
                checked += 1
    assert checked > 50


def test_overflow_is_reported():
    cfg = W.config(1)
    t, lat = cfg["target"], cfg["lattices"][0][1]
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 1 << 61)]
    assert O.solve(t, lat)["rc"] == -6


def test_fused_lattice_in_k_slabs_equals_the_whole_lattice():
    """No rewrite of a fused Spec changes k, so the fused lattice restricted to a stretch of k
    values is closed: solved against the same Matmul and bias-add + ReLU tables, each such slab
    must be the whole table's slice, entry by entry, and the counters must add up."""
    cfg = W.config(5, max_size=8)
    t = cfg["target"]
    latM, latE, latF = (lat for _, lat, _ in cfg["lattices"])
    res = O.solve_config(cfg)
    ext = res["F"]["extents"]
    full_c = res["F"]["cost"].reshape(ext)
    full_a = res["F"]["argmin"].reshape(ext)
    ks = latF["sizes"][2]
    assert ks == [1, 2, 4, 8]
    n_rw = n_adm = 0
    for lo, hi in ((0, 2), (2, 3), (3, 4)):
        slab = dict(latF, sizes=[latF["sizes"][0], latF["sizes"][1], ks[lo:hi], latF["sizes"][3]])
        r = O.solve(t, slab, deps=((latM, res["M"]["cost"]), (latE, res["E"]["cost"])))
        assert r["rc"] == 0 and r["extents"] == ext[:2] + [hi - lo] + ext[3:]
        assert np.array_equal(r["cost"].reshape(r["extents"]), full_c[:, :, lo:hi])
        assert np.array_equal(r["argmin"].reshape(r["extents"]), full_a[:, :, lo:hi])
        n_rw += r["n_rewrites"]
        n_adm += r["n_admissible"]
    assert n_rw == res["F"]["n_rewrites"] and n_adm == res["F"]["n_admissible"]
    # a k list that is no stretch of the Matmul table's is refused
    with pytest.raises(ValueError):
        O.solve(t, dict(latF, sizes=[latF["sizes"][0], latF["sizes"][1], [1, 4], latF["sizes"][3]]),
                deps=((latM, res["M"]["cost"]), (latE, res["E"]["cost"])))
