"""mrl_query_noalloc (the point query that allocates nothing: its staging is an array the library
holds in device memory) against mrl_query, through the C ABI: two calls in a row, the second with
a smaller input, so that what the first call left in the array must not show."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2505_01637_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_noalloc_query_equals_query_twice_in_a_row():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2505_01637_amd import binding as B
    cfg = W.config(3, max_size=64)
    want = O.solve_config(cfg)["M"]
    target, tabs = B.solve_config(cfg)
    tab = tabs["M"]
    ext = tab.extents
    rng = np.random.default_rng(7)

    def coords(n):
        return np.stack([rng.integers(0, e, size=n) for e in ext], axis=1).astype(np.uint32)

    # first call: as many Specs as one call takes; second call: a few, other ones
    for n in (B.NOALLOC_MAX_QUERIES, 37):
        x = coords(n)
        cost, rw = tab.query(x, noalloc=True)
        ref_cost, ref_rw = tab.query(x)
        assert np.array_equal(cost, ref_cost) and np.array_equal(rw, ref_rw)
        lin = np.ravel_multi_index(tuple(x.T.astype(np.int64)), ext)
        assert np.array_equal(cost, want["cost"][lin]) and np.array_equal(rw, want["argmin"][lin])
    # nothing at all, too many, and a coordinate outside the lattice
    cost, rw = tab.query(np.zeros((0, len(ext)), dtype=np.uint32), noalloc=True)
    assert len(cost) == 0 and len(rw) == 0
    with pytest.raises(B.MorelloError) as e:
        tab.query(coords(B.NOALLOC_MAX_QUERIES + 1), noalloc=True)
    assert e.value.code == B.E_INVAL
    bad = coords(3)
    bad[1, 2] = ext[2]
    with pytest.raises(B.MorelloError) as e:
        tab.query(bad, noalloc=True)
    assert e.value.code == B.E_RANGE
    # and the ordinary query still works afterwards
    x = coords(500)
    a, b = tab.query(x, noalloc=True), tab.query(x)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
