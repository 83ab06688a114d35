"""Pins of the oracle's lattices that take the bias-add + ReLU apart (Section 2.1: bufferize
splits a composition into a producer writing and a consumer reading a new intermediate tensor;
Section 3: a pipeline costs the sum of its stages): the bias add alone, the ReLU alone, and the
composition of the two with one bufferize per memory level of the intermediate."""
import numpy as np
import pytest

from oracle import brute_force as B
from oracle import oracle as O
from paper_2505_01637_amd import workloads as W

import util
from test_oracle_pins import brute_force_compare


def split_case(sizes, levels=2, layout=True, fused_scalar=True, fused_vec=False, s=1, caps=None, with_f=False, vec_cost=1):
    if levels == 2:
        t = W._empty_target(2, caps or (32, W.UNBOUNDED))
        t["load_coef"][1][0][0], t["store_coef"][0][1][0] = 3, 2
        t["load_coef"][1][0][1], t["store_coef"][0][1][1] = 5, 4
    else:
        t = W._empty_target(3, caps or (16, 64, W.UNBOUNDED))
        for src in range(1, 3):
            for dst in range(src):
                t["load_coef"][src][dst][0] = 2 + src - dst
                t["store_coef"][dst][src][0] = 1 + src - dst
                t["load_coef"][src][dst][1] = 4 + src - dst
                t["store_coef"][dst][src][1] = 3 + src - dst
    t["loop_overhead"] = s
    t["zero_coef"] = [1, 2, 0, 0]
    mk = [(W.MK_SCALAR_FMA, 1, 2)] if with_f else []
    if fused_scalar:
        mk.append((W.MK_SCALAR_ADDRELU, 1, 3))
    if fused_vec:
        mk.append((W.MK_VEC_ADDRELU, 2, 3))
    mk += [(W.MK_SCALAR_ADD, 1, 1), (W.MK_VEC_ADD, 2, vec_cost), (W.MK_SCALAR_RELU, 1, 1), (W.MK_VEC_RELU, 2, vec_cost)]
    t["microkernels"] = mk
    r = list(sizes)
    y = 1 if layout else 0
    lats = [("A", W._lattice(W.KIND_BIAS_ADD, [[1], r, [1], r], layout=(y, 0, y, 0, 0)), []),
            ("R", W._lattice(W.KIND_RELU, [[1], r, [1], r], layout=(y, y, 0, 0, 0)), []),
            ("S", W._lattice(W.KIND_BIAS_ADD_RELU_SPLIT, [[1], r, [1], r], layout=(y, 0, y, 0, 0)), ["A", "R"])]
    if with_f:
        lats = [("M", W._lattice(W.KIND_MATMUL_ACCUM, [[1], r, r, r], layout=(y, y, y, 0, 0)), [])] + lats
        lats.append(("F", W._lattice(W.KIND_FUSED_MM_ADD_RELU, [[1], r, r, r], layout=(y, y, 0, y, 0)), ["M", "S"]))
    return t, lats, O.solve_config({"target": t, "lattices": lats})


def test_brute_force_the_two_halves_and_the_split():
    """Every Spec of the three lattices over sizes {1, 2, 4} (two levels, both layouts) against the
    minimum over all complete programs; the programs of a bufferized Spec are enumerated through
    both stages."""
    t, lats, res = split_case([1, 2, 4])
    assert res["R"]["extents"] == [1, 3, 1, 3, 2, 2, 2, 2]
    assert res["S"]["extents"] == [1, 3, 1, 3, 2, 2, 2, 2, 2]
    assert brute_force_compare(t, lats, res, "A") == 288
    assert brute_force_compare(t, lats, res, "R") == 144
    n = brute_force_compare(t, lats, res, "S", pick=lambda s: s.dims[1] * s.dims[3] <= 2 or (s.dims[1] * s.dims[3] == 4 and sum(s.levels[:3]) <= 1))
    assert n >= 140
    ids = O.geometry(t, lats[2][1])[2]
    used = set(int(a) for a in res["S"]["argmin"])
    assert ids["bufferize"] in used or ids["bufferize"] + 1 in used


def test_brute_force_split_three_levels():
    t, lats, res = split_case([1, 2], levels=3, fused_vec=True, layout=False)
    n = brute_force_compare(t, lats, res, "S", pick=lambda s: s.dims[1] * s.dims[3] <= 2 and sum(s.levels[:3]) <= 3)
    assert n >= 45


def test_brute_force_fused_lattice_reading_the_split_table():
    """The fused Matmul -> bias add -> ReLU whose second stage may itself be bufferized: both splits
    in one program."""
    t, lats, res = split_case([1, 2], with_f=True, fused_scalar=False, layout=False)
    n = brute_force_compare(t, lats, res, "F", pick=lambda s: s.dims[1] * s.dims[2] * s.dims[3] <= 2 and sum(s.levels) <= 3)
    assert n >= 60
    # without a fused add-and-ReLU microkernel every finite entry of S goes through its bufferize somewhere below
    assert (res["S"]["cost"] != O.INF).any()


def test_split_closed_forms():
    """No loop constant, everything in level 0 (large enough): m*n scalar adds and m*n scalar
    ReLUs through the bufferize (cost 2 per element) against the fused scalar microkernel (3)."""
    t, lats, res = split_case([1, 2, 4, 8], s=0, caps=(1 << 20, W.UNBOUNDED), layout=False)
    lat = lats[2][1]
    ext = W.coord_extents(t, lat)
    c = res["S"]["cost"].reshape(ext)
    a = res["S"]["argmin"].reshape(ext)
    ids = O.geometry(t, lat)[2]
    r = lat["sizes"][1]
    for im, m in enumerate(r):
        for i_n, n in enumerate(r):
            assert int(c[0, im, 0, i_n, 0, 0, 0]) == 2 * m * n
    assert int(a[0, 0, 0, 0, 0, 0, 0]) == ids["bufferize"]            # bufferize into level 0: 1 + 1 < 3
    # in level 1 the 2-lane vector microkernels do a row of n in n/2 steps each
    for i_n, n in enumerate(r[1:], start=1):
        assert int(c[0, 0, 0, i_n, 1, 1, 1]) == 2 * (n // 2)
    assert int(a[0, 0, 0, 1, 1, 1, 1]) == ids["bufferize"] + 1        # (for n > 2 a tile of n ties, and has the lower id)
    # the halves alone
    ca = res["A"]["cost"].reshape(W.coord_extents(t, lats[0][1]))
    cr = res["R"]["cost"].reshape(W.coord_extents(t, lats[1][1]))
    assert int(ca[0, 2, 0, 3, 0, 0, 0]) == 4 * 8 and int(cr[0, 2, 0, 3, 0, 0]) == 4 * 8
    assert int(ca[0, 0, 0, 3, 1, 1, 1]) == 4 and int(cr[0, 0, 0, 3, 1, 1]) == 4
    # dearer vector microkernels than the fused scalar one per element: with a fused scalar cost of
    # 3 and vector costs of 7 per 2 lanes, level 0 still bufferizes (2 < 3), level 1 cannot use the
    # scalar ones and pays 7 * n / 2 twice
    t2, lats2, res2 = split_case([1, 2, 4, 8], s=0, caps=(1 << 20, W.UNBOUNDED), layout=False, vec_cost=7)
    c2 = res2["S"]["cost"].reshape(ext)
    assert int(c2[0, 0, 0, 3, 1, 1, 1]) == 2 * 7 * 4


def test_split_intermediate_must_fit_its_level():
    """Level 0 holds 16 bytes: a 1 x 2 Spec with in and out in level 0 (8 + 8 bytes) has no room for
    the intermediate there, so bufferize(0) does not apply and the value equals the plain kind-1
    table's; with the intermediate in level 1 the bufferize applies."""
    t, lats, res = split_case([1, 2], caps=(16, W.UNBOUNDED), layout=False, s=0)
    lat = lats[2][1]
    ext = W.coord_extents(t, lat)
    a = res["S"]["argmin"].reshape(ext)
    ids = O.geometry(t, lat)[2]
    assert int(a[0, 0, 0, 1, 0, 1, 0]) != ids["bufferize"]
    plain = dict(lat, kind=W.KIND_BIAS_ADD_RELU)
    e = O.solve(t, plain)
    # never worse than without the extra rewrite, and strictly better somewhere
    assert (res["S"]["cost"] <= e["cost"]).all() and (res["S"]["cost"] < e["cost"]).any()
    assert res["S"]["n_admissible"] == e["n_admissible"]


def test_split_rejects_wrong_tables():
    t, lats, res = split_case([1, 2])
    with pytest.raises(ValueError):
        O.solve(t, lats[2][1], deps=((lats[1][1], res["R"]["cost"]), (lats[0][1], res["A"]["cost"])))
    with pytest.raises(ValueError):
        O.solve(t, lats[2][1])
