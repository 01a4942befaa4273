"""C oracle against exhaustive shortest-path enumeration in exact rationals (N <= 12)."""
from fractions import Fraction

import numpy as np
import pytest

from helpers import tiny_graphs
from oracle import brute_force

TINY = tiny_graphs()


@pytest.mark.parametrize("name", sorted(TINY))
def test_matches_enumeration(oracle, name):
    rp, col = TINY[name]
    N = len(rp) - 1
    assert N <= 12
    D, sigma, load, per_commodity = brute_force.ewsp(rp, col)
    r = oracle.run(rp, col, want_dist=True, want_sigma=True)
    assert r.dist.tolist() == D
    assert r.sigma.tolist() == sigma
    np.testing.assert_allclose(r.load, [float(x) for x in load], rtol=1e-14)
    assert r.unreachable == sum(1 for s in range(N) for t in range(N) if D[s][t] < 0)
    assert int(r.dist_sum.sum()) == sum(x for row in D for x in row if x > 0)
    # per-commodity conservation on the enumerated flows
    src_of = np.repeat(np.arange(N), np.diff(rp))
    for (s, t), flows in per_commodity.items():
        bal = [Fraction(0)] * N
        for a, f in flows.items():
            bal[src_of[a]] -= f
            bal[int(col[a])] += f
        for v in range(N):
            assert bal[v] == (-1 if v == s else 1 if v == t else 0)


def test_enumerator_on_known_case():
    """The enumerator itself, on a case done by hand (3 paths, 2 through node 1)."""
    rp, col = TINY["asymmetric_dag"]
    D, sigma, load, per = brute_force.ewsp(rp, col)
    assert D[0][5] == 3 and sigma[0][5] == 3
    assert per[(0, 5)][0] == Fraction(2, 3) and per[(0, 5)][1] == Fraction(1, 3)
    assert D[5][0] == -1
