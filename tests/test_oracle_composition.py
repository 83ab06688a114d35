"""Pins of the oracle's lattice of two composed Matmuls (Section 2.1: a Spec may be a composition
of sub-Specs, and bufferize splits it around an intermediate tensor into a pipeline whose cost is
the sum of its stages, Section 3)."""
import numpy as np

from oracle import brute_force as B
from oracle import oracle as O
from paper_2505_01637_amd import workloads as W

import util
from test_oracle_pins import brute_force_compare


def chain_case(sizes, levels=2, layout=(0, 0, 0, 0), s=1, zero=(0, 1, 0, 0), transposed=False, caps=None):
    if levels == 2:
        t = W._empty_target(2, caps or (64, W.UNBOUNDED))
        t["load_coef"][1][0][0] = 3
        t["store_coef"][0][1][0] = 2
        if transposed:
            t["load_coef"][1][0][1] = 5
            t["store_coef"][0][1][1] = 4
    else:
        t = W._empty_target(3, caps or (32, 128, W.UNBOUNDED))
        for src in range(1, 3):
            for dst in range(src):
                t["load_coef"][src][dst][0] = 2 + src - dst
                t["store_coef"][dst][src][0] = 1 + src - dst
    t["loop_overhead"] = s
    t["zero_coef"] = list(zero)
    t["microkernels"].append((W.MK_SCALAR_FMA, 1, 1))
    r = list(sizes)
    lay_m = (layout[0] | layout[1], layout[1] | layout[2], layout[3])      # lhs, rhs, out of the Matmul table
    lats = [("M", W._lattice(W.KIND_MATMUL_ACCUM, [[1], r, r, r], layout=lay_m + (0, 0)), []),
            ("G", W._lattice(W.KIND_MATMUL_CHAIN, [r, r, r, r], layout=tuple(layout) + (0,)), ["M"])]
    return t, lats, O.solve_config({"target": t, "lattices": lats})


def test_brute_force_composition_two_levels():
    """Every Spec of the composition's lattice over sizes {1, 2} (two levels, every level
    assignment of the four operands and the intermediate) against the minimum over all complete
    programs, the two Matmul stages' programs enumerated with it."""
    t, lats, res = chain_case([1, 2])
    assert res["G"]["extents"] == [2, 2, 2, 2, 2, 2, 2, 2, 2]
    n = brute_force_compare(t, lats, res, "G", pick=lambda s: s.dims[0] * s.dims[1] * s.dims[2] * s.dims[3] <= 4)
    assert n >= 300


def test_brute_force_composition_with_layouts():
    """With layout coordinates on all four operands and transposing Moves: the Specs of one element."""
    t, lats, res = chain_case([1, 2], layout=(1, 1, 1, 1), transposed=True)
    n = brute_force_compare(t, lats, res, "G", pick=lambda s: s.dims == (1, 1, 1, 1) or
                            (s.dims in ((2, 1, 1, 1), (1, 1, 1, 2)) and sum(s.levels) <= 1))
    assert n >= 512


def test_brute_force_composition_three_levels():
    t, lats, res = chain_case([1, 2], levels=3, zero=(0, 1, 2, 0))
    n = brute_force_compare(t, lats, res, "G", pick=lambda s: (sum(s.levels) <= 6 and s.dims == (1, 1, 1, 1)) or
                            (sum(s.levels) <= 3 and s.dims[0] * s.dims[1] * s.dims[2] * s.dims[3] == 2))
    assert n >= 150


def test_composition_closed_forms():
    """Everything in registers (level 0), no loop constant, a scalar fused multiply-add of cost 1:
    the first Matmul takes m*k*p of them and the second m*p*n, whatever the order of the loops."""
    t, lats, res = chain_case([1, 2, 4, 8], s=0, zero=(0, 0, 0, 0), caps=(1 << 20, W.UNBOUNDED))
    lat = lats[1][1]
    ext = W.coord_extents(t, lat)
    c = res["G"]["cost"].reshape(ext)
    r = lat["sizes"][0]
    for ip, p in enumerate(r):
        for im, m in enumerate(r):
            for ik, k in enumerate(r):
                for i_n, n in enumerate(r):
                    assert int(c[ip, im, ik, i_n, 0, 0, 0, 0, 0]) == m * k * p + m * p * n
    # initialising the intermediate costs zero_coef[level] per element of m x p
    t2, lats2, res2 = chain_case([1, 2, 4, 8], s=0, zero=(7, 0, 0, 0), caps=(1 << 20, W.UNBOUNDED))
    c2 = res2["G"]["cost"].reshape(ext)
    # a 1 x k x p x 1 Spec has nothing to tile (m = n = 1): bufferize directly
    for ip, p in enumerate(r):
        for ik, k in enumerate(r):
            assert int(c2[ip, 0, ik, 0, 0, 0, 0, 0, 0]) == 7 * p + k * p + p
            assert int(res2["G"]["argmin"].reshape(ext)[ip, 0, ik, 0, 0, 0, 0, 0, 0]) == O.geometry(t2, lat)[2]["bufferize"]
    # tiling m to 1 first initialises the same m*p elements in total, so with s = 0 nothing is gained or lost
    assert int(c2[1, 2, 1, 1, 0, 0, 0, 0, 0]) == 7 * 4 * 2 + 4 * 2 * 2 + 4 * 2 * 2
    # tiling n recomputes the first Matmul per tile: never better than bufferizing first here
    assert int(c2[1, 0, 1, 3, 0, 0, 0, 0, 0]) == 7 * 2 + 2 * 2 + 2 * 8


def test_composition_reads_the_matmul_table():
    """With every operand and the intermediate in level 0, where nothing can move, the only
    rewrites are tiles of m and n and the bufferize: the table's value equals the minimum over
    those of the explicit formula, checked for every shape from the Matmul table's values."""
    t, lats, res = chain_case([1, 2, 4], s=3, zero=(2, 5, 0, 0), caps=(1 << 20, W.UNBOUNDED))
    latM, latG = lats[0][1], lats[1][1]
    extM, extG = W.coord_extents(t, latM), W.coord_extents(t, latG)
    cM = res["M"]["cost"].reshape(extM)
    cG = res["G"]["cost"].reshape(extG)
    r = latG["sizes"][0]
    for ip, p in enumerate(r):
        for ik in range(len(r)):
            for im, m in enumerate(r):            # ascending: the smaller shapes are checked first
                for i_n, n in enumerate(r):
                    cands = [2 * m * p + int(cM[0, im, ik, ip, 0, 0, 0]) + int(cM[0, im, ip, i_n, 0, 0, 0])]
                    for jm in range(im):
                        cands.append(m // r[jm] * int(cG[ip, jm, ik, i_n, 0, 0, 0, 0, 0]) + 3)
                    for jn in range(i_n):
                        cands.append(n // r[jn] * int(cG[ip, im, ik, jn, 0, 0, 0, 0, 0]) + 3)
                    assert int(cG[ip, im, ik, i_n, 0, 0, 0, 0, 0]) == min(cands)


def test_composition_invariants():
    """Filling from other goals first gives the same table; the admissible Specs are those whose
    operands and intermediate fit their levels."""
    t, lats, res = chain_case([1, 2, 4], levels=3, zero=(0, 1, 2, 0))
    lat = lats[1][1]
    r = res["G"]
    goals = np.random.default_rng(5).permutation(len(r["cost"]))[:300]
    again = O.solve(t, lat, deps=((lats[0][1], res["M"]["cost"]),), goals=goals)
    assert np.array_equal(again["cost"], r["cost"]) and np.array_equal(again["argmin"], r["argmin"])
    ext = W.coord_extents(t, lat)
    n_fit = 0
    for x in util.all_coords(ext):
        spec = util.spec_of_coord(t, lat, x)
        fit = B.fits(t, spec)
        n_fit += fit
        if not fit:
            assert int(r["cost"][util.linear(ext, x)]) == O.INF
    assert n_fit == r["n_admissible"]
    assert 0 < n_fit < len(r["cost"])


def test_composition_rejects_mismatched_tables():
    import pytest
    t, lats, res = chain_case([1, 2, 4])
    bad = W._lattice(W.KIND_MATMUL_CHAIN, [[1, 2], [1, 2, 4], [1, 2, 4], [1, 2, 4]])
    with pytest.raises(ValueError):
        O.solve(t, bad, deps=((lats[0][1], res["M"]["cost"]),))
    with pytest.raises(ValueError):
        O.solve(t, lats[1][1])            # no Matmul table
