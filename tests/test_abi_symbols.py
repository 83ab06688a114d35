"""The built C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import os
import re

import pytest

from paper_2505_01637_amd import binding as B
from paper_2505_01637_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "morello_mi355x.h")).read()
    declared = set(re.findall(r"\b(mrl_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_host_logic_without_gpu():
    """Descriptor validation, geometry and buffer sizes are host code."""
    cfg = W.config(5)
    t = B.Target(cfg["target"])
    want = {"M": 28094464, "E": 369664, "F": 449511424}
    for label, lat, _ in cfg["lattices"]:
        ext, n = B.geometry(t, lat)
        assert n == want[label] == W.n_specs(cfg["target"], lat)
        assert ext == W.coord_extents(cfg["target"], lat)
        cb, ab, sb = B.table_bytes(t, lat)
        assert cb == 8 * n and ab == 2 * n and sb > 0
    for number, n in [(1, 32768), (2, 16777216), (3, 92160), (4, 23708160)]:
        c = W.config(number)
        assert B.geometry(B.Target(c["target"]), c["lattices"][0][1])[1] == n
    bad = W.config(1)
    bad["target"]["n_levels"] = 7
    try:
        B.Target(bad["target"])
        assert False
    except B.MorelloError as e:
        assert e.code == B.E_INVAL
    lat = dict(cfg["lattices"][0][1])
    lat["sizes"] = [[1], [2, 4], [1], [1]]         # does not start with 1
    try:
        B.geometry(t, lat)
        assert False
    except B.MorelloError as e:
        assert e.code == B.E_INVAL and "start with 1" in str(e)


def test_unknown_dependency_is_refused_before_device_work():
    """solve_lattices finds an order by itself; a dependency that names no lattice (or a cycle)
    is refused before anything touches the device."""
    import pytest
    from paper_2505_01637_amd import workloads as W
    cfg = W.config(5, max_size=2)
    lats = [(lab, lat, ["nowhere"] if lab == "F" else deps) for lab, lat, deps in cfg["lattices"]]
    with pytest.raises(ValueError):
        B.solve_lattices(None, lats)


def test_geometry_of_every_kind_agrees_with_the_oracle():
    """Extents of every lattice kind, the parallel and the bounded ones included, from the
    library's host code and from the oracle (each derives them on its own)."""
    from oracle import oracle as O
    cases = [W.config(n, max_size=8) for n in (1, 2, 3, 4, 5, 6, 7)]
    two = W.config(1, max_size=4)
    two["target"]["capacity_bytes"][0], two["target"]["capacity_bytes"][1] = 100, W.UNBOUNDED
    two["lattices"] = [("B", dict(two["lattices"][0][1], kind=W.KIND_MATMUL_BOUNDED), [])]
    cases.append(two)
    for cfg in cases:
        t = B.Target(cfg["target"])
        for label, lat, _ in cfg["lattices"]:
            ext, n = B.geometry(t, lat)
            oext, _, _ = O.geometry(cfg["target"], lat)
            assert ext == oext == W.coord_extents(cfg["target"], lat), (cfg["name"], label)
    # a capacity of 100 bytes gives the bounds 0, 1, 2, ..., 64: eight values; the unbounded level has no axis
    assert B.geometry(B.Target(two["target"]), two["lattices"][0][1])[0][-1] == 8
    # a parallel lattice needs at least one thread
    bad = W.config(6, max_size=4)
    bad["target"]["threads"] = 0
    try:
        B.geometry(B.Target(bad["target"]), bad["lattices"][1][1])
        assert False
    except B.MorelloError as e:
        assert e.code == B.E_INVAL


def test_move_coefficients_whose_sum_exceeds_32_bits_are_refused():
    """The accumulated output of a Matmul pays load + store per element; the library keeps that sum
    in 32 bits and says so when it does not fit (no silent wrap-around)."""
    cfg = W.config(1, max_size=4)
    cfg["target"]["load_coef"][1][0][0] = (1 << 32) - 1
    cfg["target"]["store_coef"][0][1][0] = 1
    try:
        B.geometry(B.Target(cfg["target"]), cfg["lattices"][0][1])
        assert False
    except B.MorelloError as e:
        assert e.code == B.E_INVAL and "too large" in str(e)
    cfg["target"]["store_coef"][0][1][0] = 0        # no store: the output cannot move, the inputs can
    B.geometry(B.Target(cfg["target"]), cfg["lattices"][0][1])


def test_graph_call_refuses_malformed_graphs_before_device_work():
    """mrl_solve_graph: deps are indices of earlier jobs, every job has a stream of its own, 1..16 jobs."""
    import ctypes as C
    cfg = W.config(5, max_size=2)
    t = B.Target(cfg["target"])
    descs = [B._lattice_desc(lat) for _, lat, _ in cfg["lattices"]]
    def call(n, deps=((), (), (0, 1)), streams=(1, 2, 3)):
        jobs = (B._Job * 17)()
        for i in range(3):
            jobs[i].lattice = C.cast(C.pointer(descs[i]), C.c_void_p)
            jobs[i].n_deps = len(deps[i])
            for k, d in enumerate(deps[i]):
                jobs[i].deps[k] = d
            jobs[i].d_cost = jobs[i].d_argmin = jobs[i].d_scratch = 256      # never dereferenced here
            jobs[i].scratch_bytes = 0
            jobs[i].hip_stream = streams[i]
        out = (C.c_void_p * 17)()
        rc = B.lib().mrl_solve_graph(t._h, jobs, C.c_uint32(n), out, None)
        assert all(not h for h in out)
        return rc, B.lib().mrl_last_error().decode()
    assert call(0)[0] == B.E_INVAL
    assert call(17)[0] == B.E_INVAL
    rc, msg = call(3, deps=((), (1,), (0, 1)))
    assert rc == B.E_INVAL and "earlier job" in msg
    rc, msg = call(3, deps=((), (), (0, 2)))
    assert rc == B.E_INVAL and "earlier job" in msg
    rc, msg = call(3, streams=(1, 2, 1))
    assert rc == B.E_INVAL and "share a stream" in msg
    descs[1] = descs[0]                 # the same lattice twice
    rc, msg = call(3)
    assert rc == B.E_INVAL and "same lattice" in msg


def test_moves_as_specs_host_checks():
    """Host-side checks (no device work): geometry of a MOVE lattice, and what a MOVE or
    MATMUL_MOVES lattice is refused for."""
    import ctypes as C
    from paper_2505_01637_amd import binding as B
    from paper_2505_01637_amd import workloads as W
    from oracle import oracle as O
    t = W._empty_target(3, (64, 128, W.UNBOUNDED))
    t["line_bytes"] = 8
    t["microkernels"] = [(W.MK_SCALAR_MOVE, 1, 3), (W.MK_VECTOR_MOVE, 2, 2)]
    r = [1, 2, 3, 4, 6, 8]
    lat = W._lattice(W.KIND_MOVE, [[1], r, [1], r], layout=(1, 1, 0, 0, 0), dtype=(1, 0, 0, 0, 0))
    target = B.Target(t)
    ext, n = B.geometry(target, lat)
    want_ext, _, _ = O.geometry(t, lat)
    assert ext == want_ext == [1, 6, 1, 6, 3, 3, 3, 2, 3, 2, 2, 2, 2]
    assert n == W.n_specs(t, lat)
    for bad_target, bad_lat in ((dict(t, line_bytes=0), lat),
                                (t, W._lattice(W.KIND_MOVE, [[1], r, r, r])),
                                (t, W._lattice(W.KIND_MATMUL_MOVES, [[1, 2], r, r, r]))):
        with pytest.raises(B.MorelloError) as e:
            B.geometry(B.Target(bad_target), bad_lat)
        assert e.value.code == B.E_INVAL
