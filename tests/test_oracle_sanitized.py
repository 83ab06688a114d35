"""The C oracle built with -fsanitize=address,undefined and run over small lattices of every
kind: no report from either sanitizer, and the same tables, counters and box lists as the
ordinary build.  (The oracle is index arithmetic over malloc'ed tables; a stray access that
happens to read plausible memory would otherwise go unnoticed.)"""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2505_01637_amd import workloads as W


@pytest.fixture(scope="module")
def exe(tmp_path_factory):
    return O.build_sanitized(str(tmp_path_factory.mktemp("sanitized")))


def bounded_pipeline():
    """Two levels of finite capacity; Matmul, bias-add + ReLU and fused tables, all with memory bounds."""
    t = W._empty_target(2, (16, 64))
    t["load_coef"][1][0][0], t["store_coef"][0][1][0] = 3, 5
    t["loop_overhead"] = 1
    t["zero_coef"] = [1, 2, 0, 0]
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 2), (W.MK_SCALAR_ADDRELU, 1, 1), (W.MK_VEC_ADDRELU, 2, 1)]
    r = [1, 2]
    return {"name": "bounded pipeline", "target": t,
            "lattices": [("M", W._lattice(W.KIND_MATMUL_BOUNDED, [[1], r, r, r]), []),
                         ("E", W._lattice(W.KIND_BIAS_ADD_RELU_BOUNDED, [[1], r, [1], r]), []),
                         ("F", W._lattice(W.KIND_FUSED_BOUNDED, [[1], r, r, r]), ["M", "E"])]}


def matmul_with_move_specs():
    """A lattice of Move Specs and a Matmul lattice whose Moves are looked up in it."""
    t = W._empty_target(3, (64, 128, W.UNBOUNDED))
    t["loop_overhead"] = 1
    t["line_bytes"] = 8
    t["level_weight"] = [1, 2, 5, 0]
    t["microkernels"] = [(W.MK_SCALAR_FMA, 1, 1), (W.MK_SCALAR_MOVE, 1, 3), (W.MK_VECTOR_MOVE, 2, 2),
                         (W.MK_VECTOR_MOVE_ALIGNED, 2, 1)]
    r = [1, 2, 4]
    return {"name": "moves", "target": t,
            "lattices": [("V", W._lattice(W.KIND_MOVE, [[1], r, [1], r], layout=(1, 1, 0, 0, 0), dtype=(1, 1, 0, 0, 0)), []),
                         ("M", W._lattice(W.KIND_MATMUL_MOVES, [[1], r, r, r], layout=(1, 0, 1, 0, 0), dtype=(1, 0, 0, 0, 0),
                                          base_bytes=(2, 4, 4, 4, 4)), ["V"])]}


@pytest.mark.parametrize("number,max_size", [(1, 6), (3, 16), (4, 2), (5, 4), (6, 4), (7, 1), (8, None), (9, None), (10, 2), (11, 2), (12, 4)])
def test_sanitized_oracle_agrees_with_the_ordinary_build(exe, tmp_path, number, max_size):
    cfg = bounded_pipeline() if number == 8 else matmul_with_move_specs() if number == 9 else W.config(number, max_size=max_size)
    got = O.run_sanitized(exe, cfg, str(tmp_path))
    want = O.solve_config(cfg)
    for label, lat, _ in cfg["lattices"]:
        g, w = got[label], want[label]
        assert g["rc"] == w["rc"] == 0
        assert np.array_equal(g["cost"], w["cost"]) and np.array_equal(g["argmin"], w["argmin"])
        assert g["n_admissible"] == w["n_admissible"]
        # the driver solves one goal before the sweep; the count of rewrites does not depend on the order
        assert g["n_rewrites"] == w["n_rewrites"]
        dec, cst = O.compress_table(cfg["target"], lat, w["cost"], w["argmin"])
        assert g["decision_boxes"].tobytes() == dec.tobytes()
        assert g["cost_boxes"].tobytes() == cst.tobytes()


def test_sanitized_oracle_reports_overflow(exe, tmp_path):
    """Costs past 2^62: the range check itself must not overflow (128-bit intermediates)."""
    cfg = W.config(2, max_size=4)
    cfg["target"]["microkernels"] = [(W.MK_SCALAR_FMA, 1, 1 << 61)]
    got = O.run_sanitized(exe, cfg, str(tmp_path))
    assert got["M"]["rc"] == -6
    assert got["M"]["rc"] == O.solve_config(cfg)["M"]["rc"]
