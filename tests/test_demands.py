"""Commodities of unequal demand.  The paper's commodities all have the same demand (Sec. 3.1.1); with
demand(s,t) the equal split over shortest paths (Sec. 5.2) gives
load[a] = sum_{s,t} demand(s,t) * (#shortest s->t paths through a) / sigma(s,t).
CPU: the oracle against exact path enumeration, closed forms and invariants; GPU: a2a_link_loads_demand
against the oracle on seeded demand matrices."""
from fractions import Fraction

import numpy as np
import pytest

from a2a_inputs import topologies as gen
from helpers import tiny_graphs


def seeded_demand(n_src, N, seed, zero_every=5):
    """Whole-number demands 0..7 from the shared LCG stream, about one in `zero_every` of them zero."""
    st = gen.lcg_stream(seed)
    d = np.empty((n_src, N), dtype=np.float64)
    for s in range(n_src):
        for t in range(N):
            x = next(st)
            d[s, t] = 0.0 if x % zero_every == 0 else float(1 + (x >> 8) % 7)
    return d


# ---------------------------------------------------------------------------------------------------------
# CPU: the oracle
# ---------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name", sorted(tiny_graphs()))
def test_against_path_enumeration(oracle, name):
    """Every shortest path written out, each commodity's demand split equally over them, in exact fractions."""
    from oracle import brute_force
    rp, col = tiny_graphs()[name]
    N = len(rp) - 1
    dem = seeded_demand(N, N, 31 + N)
    D, sigma, _, per = brute_force.ewsp(rp, col)
    want = [Fraction(0)] * len(col)
    wd = Fraction(0)
    for (s, t), flows in per.items():
        w = Fraction(int(dem[s, t]))
        wd += w * D[s][t]
        for a, f in flows.items():
            want[a] += w * f
    load, got_wd = oracle.run_demand(rp, col, dem)
    np.testing.assert_allclose(load, [float(x) for x in want], rtol=1e-13, atol=0)
    assert got_wd == pytest.approx(float(wd), rel=1e-14)


def test_unit_demand_is_the_unit_function(oracle):
    for rp, col in (gen.torus([4, 5]), gen.imase_itoh(50, 3), gen.random_regular(60, 3, 9)):
        N = len(rp) - 1
        r = oracle.run(rp, col)
        load, wd = oracle.run_demand(rp, col, np.ones((N, N)))
        assert np.array_equal(load, r.load)
        assert wd == float(r.dist_sum.sum())


def test_linear_in_the_demands(oracle):
    rp, col = gen.random_regular(40, 3, 4)
    N = len(rp) - 1
    d1, d2 = seeded_demand(N, N, 1), seeded_demand(N, N, 2)
    l1, w1 = oracle.run_demand(rp, col, d1)
    l2, w2 = oracle.run_demand(rp, col, d2)
    l12, w12 = oracle.run_demand(rp, col, d1 + 4.0 * d2)
    np.testing.assert_allclose(l12, l1 + 4.0 * l2, rtol=1e-13)
    assert w12 == pytest.approx(w1 + 4.0 * w2, rel=1e-14)


def test_one_commodity_on_a_directed_ring(oracle):
    """One path per pair: demand(s, s+k) rides the k links s -> s+1 -> ... -> s+k and no other."""
    N = 9
    rp, col = gen.ring(N)
    dem = np.zeros((N, N))
    dem[2, 6] = 5.0   # links 2,3,4,5
    dem[7, 1] = 0.25  # links 7,8,0
    load, wd = oracle.run_demand(rp, col, dem)
    want = np.zeros(N)
    want[[2, 3, 4, 5]] += 5.0
    want[[7, 8, 0]] += 0.25
    assert np.array_equal(load, want)  # link i is i -> i+1
    assert wd == 5.0 * 4 + 0.25 * 3


def test_antipodal_pair_splits_in_two(oracle):
    """Bidirectional ring of 8: the two shortest 0 -> 4 paths go round either side, half the demand each."""
    rp, col = gen.bidirectional_ring(8)
    dem = np.zeros((8, 8))
    dem[0, 4] = 3.0
    load, wd = oracle.run_demand(rp, col, dem)
    assert wd == 12.0
    for u in range(8):
        for a in range(rp[u], rp[u + 1]):
            w = int(col[a])
            clockwise = w == (u + 1) % 8 and u in (0, 1, 2, 3)
            counter = w == (u - 1) % 8 and u in (0, 7, 6, 5)
            assert load[a] == (1.5 if clockwise or counter else 0.0), (u, w)


@pytest.mark.parametrize("make", [lambda: gen.torus([3, 5]), lambda: gen.imase_itoh(40, 3),
                                  lambda: gen.csr_from_rows([[1], [2], [0, 3], [0], [0], []])])
def test_conservation_and_total(oracle, make):
    """Per node: what leaves minus what enters = demand it sends minus demand it receives (reachable pairs);
    all links together carry demand x distance."""
    rp, col = make()
    N = len(rp) - 1
    dem = seeded_demand(N, N, 77)
    np.fill_diagonal(dem, 0.0)
    dist = oracle.run(rp, col, want_dist=True).dist
    ok = dist > 0
    load, wd = oracle.run_demand(rp, col, dem)
    assert load.sum() == pytest.approx(float((dem * dist)[ok].sum()), rel=1e-13)
    assert wd == pytest.approx(float((dem * dist)[ok].sum()), rel=1e-14)
    out = np.array([load[rp[v]:rp[v + 1]].sum() for v in range(N)])
    inn = np.zeros(N)
    np.add.at(inn, col, load)
    sent = np.where(ok, dem, 0.0).sum(axis=1)
    recv = np.where(ok, dem, 0.0).sum(axis=0)
    np.testing.assert_allclose(out - inn, sent - recv, rtol=0, atol=1e-9)


def test_partial_source_range_and_bad_arguments(oracle):
    rp, col = gen.torus([4, 4])
    N = 16
    dem = seeded_demand(N, N, 5)
    full, wfull = oracle.run_demand(rp, col, dem)
    a, wa = oracle.run_demand(rp, col, dem[:6], 0)
    b, wb = oracle.run_demand(rp, col, dem[6:], 6)
    np.testing.assert_allclose(a + b, full, rtol=1e-14)
    assert wa + wb == pytest.approx(wfull, rel=1e-15)
    with pytest.raises(ValueError):
        oracle.run_demand(rp, col, dem[:, :5])
    with pytest.raises(ValueError):
        oracle.run_demand(rp, col, dem, 3)  # 3 + 16 sources > N
