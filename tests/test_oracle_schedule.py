"""Schedule extraction of the oracle (Section 4: follow the memoized rewrites; Figure 1: the
program they spell out), pinned by evaluating Section 3's cost equation on the extracted tree
with the brute-force module's evaluator: it must give back the table's entry of the goal."""
import numpy as np
import pytest

from oracle import brute_force as BF
from oracle import oracle as O
from oracle import schedule as S
from paper_2505_01637_amd import workloads as W



def check_tree(tree, results):
    """Every node's cost is the table's entry of its Spec and the cost of its subtree; leaves are
    microkernels; a loop has one child, a Move one, a pipeline two."""
    n = 0
    stack = [tree]
    while stack:
        t = stack.pop()
        n += 1
        assert S.tree_cost(t) == t["cost"]
        tag = t["node"][0]
        if tag == "alloc" and t["label"] == "M" and any(ch["label"] == "V" for ch in t["children"]):
            # an alloc-binding whose Moves are Specs: load (unless only written), body, store (if written)
            labels = [ch["label"] for ch in t["children"]]
            assert labels in (["V", "M"], ["V", "M", "V"])
        else:
            assert len(t["children"]) == {"mk": 0, "loop": 1, "alloc": 1, "pipeline": 2}[tag]
        stack += t["children"]
    return n


def sample_goals(results, label, k, seed):
    cost = results[label]["cost"]
    finite = np.flatnonzero(cost != np.uint64(O.INF))
    rng = np.random.default_rng(seed)
    picks = rng.choice(finite, size=min(k, len(finite)), replace=False)
    ext = [int(e) for e in results[label]["extents"]]
    return [tuple(int(v) for v in np.unravel_index(int(p), ext)) for p in picks]


@pytest.mark.parametrize("number,max_size", [(1, None), (2, 8), (3, 64), (4, 8)])
def test_extracted_program_costs_what_the_table_says(number, max_size):
    cfg = W.config(number, max_size=max_size)
    res = O.solve_config(cfg)
    label = cfg["lattices"][0][0]
    nodes = 0
    for goal in sample_goals(res, label, 200, seed=number):
        tree = S.extract(cfg["target"], cfg["lattices"], res, label, goal)
        assert tree["coord"] == goal
        nodes += check_tree(tree, res)
    assert nodes > 400


def test_fused_program_has_both_parts():
    cfg = W.config(5, max_size=8)
    res = O.solve_config(cfg)
    seen_pipeline = 0
    for goal in sample_goals(res, "F", 300, seed=5):
        tree = S.extract(cfg["target"], cfg["lattices"], res, "F", goal)
        check_tree(tree, res)
        flat = S.preorder(tree)
        labels = {n[0] for n in flat}
        if "M" in labels or "E" in labels:
            assert {"M", "E"} <= labels          # bufferize brings both
            seen_pipeline += 1
    assert seen_pipeline > 0


def test_goal_without_implementation():
    cfg = W.config(2, max_size=64)
    res = O.solve_config(cfg)
    cost = res["M"]["cost"]
    bad = int(np.flatnonzero(cost == np.uint64(O.INF))[0])
    ext = [int(e) for e in res["M"]["extents"]]
    with pytest.raises(ValueError):
        S.extract(cfg["target"], cfg["lattices"], res, "M", tuple(int(v) for v in np.unravel_index(bad, ext)))


def test_figure_1_goal():
    """The worked example's target and goal (Figure 1): the extracted program is the hand-derived
    optimum of the fixture -- move the whole output to VRF, loop over m, loop over k, then
    BroadcastVecMultAdd -- and costs 293, below the 1061 of the schedule the figure spells out."""
    from test_oracle_pins import fig1_setup
    g, t, lat = fig1_setup()
    res = {"M": O.solve(t, lat)}
    goal_spec = BF.Spec(0, (1, 4, 4, 16), (0, 1, 2, 0, 0), (0,) * 5, (0,) * 5)
    goal = S.coord_of_spec(lat, goal_spec)
    tree = S.extract(t, [("M", lat, [])], res, "M", goal)
    assert S.tree_cost(tree) == tree["cost"] == g["optimum_cost"] == 293
    assert tree["cost"] <= g["figure1_schedule_cost"]
    tags = [n["node"][0] for n in _chain(tree)]
    assert tags == ["alloc", "loop", "loop", "mk"]
    costs = [n["cost"] for n in _chain(tree)]
    assert costs == [293, 37, 9, 2]           # the fixture's optimum_derivation, outermost first


def _chain(tree):
    out = [tree]
    while out[-1]["children"]:
        assert len(out[-1]["children"]) == 1
        out.append(out[-1]["children"][0])
    return out


def test_programs_with_move_specs():
    """Section 2, Memory Movement: the alloc-binding of an operand holds its load Move Spec, the
    body and (for the accumulated output) its store Move Spec, each implemented like any Spec;
    the extracted tree costs what the table says, down through the Move Specs' own loops and
    move microkernels, also with packed layouts."""
    for number, size in ((9, 8), (12, 8)):
        cfg = W.config(number, max_size=size)
        res = O.solve_config(cfg)
        nodes = with_moves = 0
        for goal in sample_goals(res, "M", 120, seed=number):
            tree = S.extract(cfg["target"], cfg["lattices"], res, "M", goal)
            nodes += check_tree(tree, res)
            with_moves += any(n[0] == "V" for n in S.preorder(tree))
        assert nodes > 400 and with_moves > 20
        for goal in sample_goals(res, "V", 120, seed=number):
            tree = S.extract(cfg["target"], cfg["lattices"], res, "V", goal)
            check_tree(tree, res)
            assert {n[0] for n in S.preorder(tree)} == {"V"}
