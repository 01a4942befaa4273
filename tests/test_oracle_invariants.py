"""Invariants that hold for EwSP loads on any topology (checked on the C oracle)."""
import numpy as np
import pytest

import a2a_inputs as gen
from helpers import tiny_graphs

GRAPHS = {
    "torus5x4": lambda: gen.torus([5, 4]),
    "kautz_100_3": lambda: gen.imase_itoh(100, 3),
    "kautz_81_8": lambda: gen.imase_itoh(81, 8),
    "rr_300_4": lambda: gen.random_regular(300, 4, 5),
    "rr_257_8": lambda: gen.random_regular(257, 8, 11),
    "punctured_333": lambda: gen.remove_arcs(gen.torus([3, 3, 3]), [3, 50, 101]),
    "punctured_nodes_333": lambda: gen.remove_nodes(gen.torus([3, 3, 3]), [0, 13, 20]),
}
GRAPHS.update({k: (lambda v=v: v) for k, v in tiny_graphs().items()})


@pytest.mark.parametrize("name", sorted(GRAPHS))
def test_per_source_flow_conservation_and_level_cuts(oracle, name):
    rp, col = GRAPHS[name]()
    N = len(rp) - 1
    src = np.repeat(np.arange(N), np.diff(rp))
    total = np.zeros(len(col))
    for s in range(N):
        r = oracle.run(rp, col, s, 1, want_dist=True, want_sigma=True)
        d = r.dist[0]
        reach = d >= 0
        inflow = np.bincount(col, weights=r.load, minlength=N)
        outflow = np.bincount(src, weights=r.load, minlength=N)
        # the source emits one unit per reachable destination; every other reachable node
        # absorbs exactly one unit (source-based conservation of the decomposed master
        # LP, Sec. 3.1.1, met with equality at F = 1)
        assert outflow[s] == pytest.approx(reach.sum() - 1, rel=1e-12)
        assert inflow[s] == 0
        others = reach.copy(); others[s] = False
        np.testing.assert_allclose((inflow - outflow)[others], 1.0, rtol=1e-12, atol=1e-12)
        assert np.all(r.load[~reach[src]] == 0)
        # only links one level apart carry flow
        on_dag = reach[src] & (d[col] == d[src] + 1)
        assert np.all(r.load[~on_dag] == 0)
        assert np.all(r.load[on_dag] > 0)
        # flow crossing level l-1 -> l = number of nodes at distance >= l
        for lvl in range(1, int(d.max()) + 1):
            cut = r.load[on_dag & (d[col] == lvl)].sum()
            assert cut == pytest.approx(np.sum(d >= lvl), rel=1e-12)
        total += r.load
    full = oracle.run(rp, col, threads=3)
    np.testing.assert_allclose(full.load, total, rtol=1e-13)
    # every unit of demand uses D(s,t) link-units
    assert full.load.sum() == pytest.approx(float(full.dist_sum.sum()), rel=1e-12)
    if len(col):
        b = oracle.bound(rp, full.load, int(full.dist_sum.sum()))
        assert b["max_load"] * len(col) >= full.dist_sum.sum() * (1 - 1e-12)


def test_thread_count_does_not_change_integers(oracle):
    rp, col = gen.random_regular(1000, 5, 3)
    a = oracle.run(rp, col, threads=1, want_dist=True, want_sigma=True)
    b = oracle.run(rp, col, threads=7, want_dist=True, want_sigma=True)
    assert np.array_equal(a.dist, b.dist) and np.array_equal(a.sigma, b.sigma)
    assert np.array_equal(a.dist_sum, b.dist_sum) and a.unreachable == b.unreachable
    np.testing.assert_allclose(a.load, b.load, rtol=1e-13)


def test_source_range_rows(oracle):
    rp, col = gen.torus([4, 5])
    whole = oracle.run(rp, col, want_dist=True, want_sigma=True)
    part = oracle.run(rp, col, 7, 5, want_dist=True, want_sigma=True, threads=2)
    assert np.array_equal(part.dist, whole.dist[7:12])
    assert np.array_equal(part.sigma, whole.sigma[7:12])
    assert np.array_equal(part.dist_sum, whole.dist_sum[7:12])


def test_c5_sampled_sources(oracle):
    """No closed form at C5: distance sums obey the tree-fill bound, loads obey conservation."""
    rp, col = gen.named_config("C5")
    N = 65536
    r = oracle.run(rp, col, 1000, 16, threads=8, want_dist=True)
    left, lvl, smin = N - 1, 1, 0
    while left > 0:
        take = min(left, 8 ** lvl); smin += lvl * take; left -= take; lvl += 1
    assert smin == 350418
    assert r.unreachable == 0 and np.all(r.dist_sum >= smin)
    assert r.dist.max() <= 8
    assert r.load.sum() == pytest.approx(float(r.dist_sum.sum()), rel=1e-12)


def test_rejects_bad_ranges(oracle):
    rp, col = gen.ring(5)
    with pytest.raises(ValueError):
        oracle.run(rp, col, 3, 4)
    with pytest.raises(ValueError):
        oracle.run(rp, col, -1, 2)
