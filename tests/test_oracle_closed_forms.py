"""Pins of the C oracle against what the paper prints and what mathematics fixes."""
import math
from fractions import Fraction

import numpy as np
import pytest

import a2a_inputs as gen
from helpers import paper_values, frac


def full(oracle, csr, **kw):
    return oracle.run(csr[0], csr[1], threads=8, want_dist=True, want_sigma=True, **kw)


def test_torus333_matches_paper_flow_value(oracle):
    """Sec. 5.1: the 3x3x3 torus carries concurrent flow 1/9; Sec. 5.3: all-to-all time = max
    link load = 1/flow.  The torus is arc-transitive, so EwSP loads every link equally."""
    f = frac(paper_values()["torus333_flow_value"])
    csr = gen.torus([3, 3, 3])
    r = full(oracle, csr)
    assert r.load.shape == (162,)
    np.testing.assert_allclose(r.load, float(1 / f), rtol=1e-12)
    assert int(r.dist_sum.sum()) == 27 * 54
    b = oracle.bound(csr[0], r.load, int(r.dist_sum.sum()))
    assert b["flow_value"] == pytest.approx(float(f), rel=1e-12)
    assert b["ratio"] == pytest.approx(1.0, rel=1e-12)


def test_throughput_upper_bound_formula(oracle):
    """Sec. 5.1 prints (N-1) f b = 26 * (2/27) * 3.125 = 6.01 GB/s.  Drive the oracle's formula
    with a load vector whose maximum is 1/f = 13.5."""
    pv = paper_values()
    N = int(pv["upper_bound_N"]); f = frac(pv["upper_bound_f"]); b = float(pv["upper_bound_b_GBps"])
    csr = gen.torus([3, 3, 3])
    load = np.full(162, 1.0); load[17] = float(1 / f)
    out = oracle.bound(csr[0], load, 1458, m=1.0, b=b)
    assert N == 27 and out["argmax_arc"] == 17
    # the exact product is 6.0185...; the paper prints it cut to two decimals
    assert math.floor(out["throughput_upper"] * 100) / 100 == float(pv["upper_bound_GBps"])
    # throughput (N-1) m / T with T = Lmax m / b is the same number (Sec. 2.2)
    assert out["throughput"] == pytest.approx(out["throughput_upper"], rel=1e-14)


@pytest.mark.parametrize("dims", [[8, 8], [5, 4], [16, 16, 16], [7], [6, 3, 4]])
def test_torus_closed_forms(oracle, dims):
    """Ring of k nodes: sum_t D = floor(k^2/4); dimensions add.  sigma = multinomial of the
    per-dimension offsets, doubled for every dimension at offset k/2."""
    csr = gen.torus(dims)
    N = int(np.prod(dims))
    r = full(oracle, csr)
    per_node = sum((k * k // 4) * (N // k) for k in dims)
    assert np.all(r.dist_sum == per_node)
    assert r.unreachable == 0 and r.flags == 0
    # distance / sigma of every pair from closed form
    ids = np.arange(N)
    coords = []
    s = 1
    for k in dims:
        coords.append((ids // s) % k); s *= k
    for src in (0, N // 3, N - 1):
        offs = []
        for a, k in enumerate(dims):
            o = (coords[a] - coords[a][src]) % k
            offs.append(np.minimum(o, k - o))
        D = sum(offs)
        assert np.array_equal(r.dist[src], D)
        for t in (1, N // 2, N - 2, (src + 7) % N):
            o = [int(x[t]) for x in offs]
            sig = math.factorial(sum(o))
            for a, k in enumerate(dims):
                sig //= math.factorial(o[a])
                if k % 2 == 0 and o[a] == k // 2:
                    sig *= 2
            assert int(r.sigma[src, t]) == sig
    if len(set(dims)) == 1:  # arc-transitive: every link carries per-node sumD / d
        np.testing.assert_allclose(r.load, per_node / (2 * len(dims)), rtol=1e-12)


def test_c1_and_c3_values(oracle):
    r = full(oracle, gen.named_config("C1"))
    assert np.all(r.dist_sum == 256) and int(r.sigma.max()) == 280
    np.testing.assert_allclose(r.load, 64.0, rtol=1e-12)
    r = oracle.run(*gen.named_config("C3"), threads=8, want_sigma=True)
    assert np.all(r.dist_sum == 49152)
    assert int(r.sigma.max()) == math.factorial(24) // math.factorial(8) ** 3 * 8 == 75724094160
    np.testing.assert_allclose(r.load, 8192.0, rtol=1e-12)


@pytest.mark.parametrize("n", [1, 3, 6, 10])
def test_hypercube_closed_forms(oracle, n):
    """D = popcount(s xor t); sigma = D!; per-node sum D = n 2^(n-1); each link load 2^(n-1)."""
    csr = gen.hypercube(n)
    N = 1 << n
    r = full(oracle, csr)
    x = np.arange(N)[:, None] ^ np.arange(N)[None, :]
    pc = np.zeros_like(x)
    for k in range(n):
        pc += (x >> k) & 1
    assert np.array_equal(r.dist, pc)
    fact = np.array([math.factorial(i) for i in range(n + 1)], dtype=np.uint64)
    assert np.array_equal(r.sigma, fact[pc])
    assert np.all(r.dist_sum == n * 2 ** (n - 1))
    np.testing.assert_allclose(r.load, 2.0 ** (n - 1), rtol=1e-12)


def test_k44_fractional_loads(oracle):
    """K4,4: 4 neighbours at distance 1, 3 same-side nodes at distance 2 over 4 paths each.
    Per link: 1 + 3*(1/4) outbound first hops + 3*(1/4) second hops = 2.5."""
    csr = gen.complete_bipartite(4)
    r = full(oracle, csr)
    assert int(r.dist_sum.sum()) == 80
    assert np.array_equal(r.load, np.full(32, 2.5))
    assert int(r.sigma[0, 1]) == 4 and int(r.sigma[0, 4]) == 1


@pytest.mark.parametrize("N", [2, 5, 64, 131])
def test_directed_ring(oracle, N):
    """Unique paths: D = (t - s) mod N, every link carries N(N-1)/2."""
    r = full(oracle, gen.ring(N))
    D = (np.arange(N)[None, :] - np.arange(N)[:, None]) % N
    assert np.array_equal(r.dist, D)
    assert np.all(r.sigma == 1)
    assert np.array_equal(r.load, np.full(N, N * (N - 1) / 2.0))


def test_asymmetric_per_path_split(oracle):
    """Per-path (not per-next-hop) splitting: link 0->1 carries 2/3 of commodity (0,5)."""
    from helpers import ASYMMETRIC_ROWS
    csr = gen.csr_from_rows(ASYMMETRIC_ROWS)
    r = oracle.run(csr[0], csr[1], 0, 1, want_sigma=True, want_dist=True)
    assert list(r.sigma[0]) == [1, 1, 1, 1, 2, 3]
    # link ids: 0:(0,1) 1:(0,2) 2:(1,3) 3:(1,4) 4:(2,4) 5:(3,5) 6:(4,5)
    expect = [1 + 1 + Fraction(1, 2) + Fraction(2, 3), 1 + Fraction(1, 2) + Fraction(1, 3),
              1 + Fraction(1, 3), Fraction(1, 2) + Fraction(1, 3), Fraction(1, 2) + Fraction(1, 3),
              Fraction(1, 3), Fraction(2, 3)]
    np.testing.assert_allclose(r.load, [float(x) for x in expect], rtol=1e-15)


def test_parallel_arcs_are_distinct_links(oracle):
    csr = gen.csr_from_rows([[1, 1], [2], [0]])
    r = full(oracle, csr)
    assert int(r.sigma[0, 1]) == 2 and int(r.sigma[0, 2]) == 2 and int(r.sigma[2, 1]) == 2
    # links 0,1 (0->1 twice) share: pairs (0,1),(0,2),(2,1) each 1/2 per copy
    np.testing.assert_allclose(r.load, [1.5, 1.5, 3.0, 3.0], rtol=1e-15)


def test_unreachable_and_flags(oracle):
    csr = gen.csr_from_rows([[1], [2], [0, 3], [0], [0], []])
    r = full(oracle, csr)
    assert r.dist[0, 4] == -1 and r.dist[0, 5] == -1 and r.dist[5, 0] == -1 and r.dist[4, 3] == 4
    assert r.sigma[0, 4] == 0
    # node 5 reaches nothing (5), nothing reaches 5 (5), nothing but 4 reaches 4 (4)
    assert r.unreachable == 5 + 5 + 4
    assert r.flags == 2


def test_sigma_overflow_flag(oracle):
    """A chain of 54 two-link stages has 2^54 shortest end-to-end paths."""
    rows = [[i + 1, i + 1] for i in range(54)] + [[]]
    csr = gen.csr_from_rows(rows)
    r = oracle.run(csr[0], csr[1], 0, 1, want_sigma=True)
    assert int(r.sigma[0, 52]) == 2 ** 52 and int(r.sigma[0, 54]) == 2 ** 54
    assert r.flags & 1
    r = oracle.run(csr[0], csr[1], 2, 1, want_sigma=True)
    assert not (r.flags & 1)


def test_thm1_closed_form_and_fill_bound(oracle):
    """Proof of Theorem 1: a source's distance sum is at least that of a tree with d^l nodes
    at level l; for a full k-layer tree it equals (d^(k+1)(k-1) - d^k k + d)/(d-1)^2."""
    def full_tree(d, k):
        return eval(paper_values()["thm1_formula"], {"d": d, "k": k})
    assert full_tree(2, 3) == 10 == 0 * 1 + 1 * 2 + 2 * 4
    for d, k in [(3, 4), (4, 7), (8, 5)]:
        assert full_tree(d, k) == sum(i * d ** i for i in range(k))

    def s_min(N, d):
        left, lvl, tot = N - 1, 1, 0
        while left > 0:
            take = min(left, d ** lvl)
            tot += lvl * take; left -= take; lvl += 1
        return tot
    assert s_min((4 ** 7 - 1) // 3, 4) == full_tree(4, 7)
    # generalized Kautz graphs come close to the bound (Sec. 5.4): here one source meets it
    csr = gen.imase_itoh(16384, 4)
    r = oracle.run(csr[0], csr[1], threads=8, want_sigma=True)
    assert int(r.dist_sum.min()) == s_min(16384, 4) == 107409
    assert np.all(r.dist_sum >= 107409)
    # N = 4^7: unique shortest paths, so loads are whole numbers
    assert int(r.sigma.max()) == 1
    assert np.array_equal(r.load, np.round(r.load))
    assert r.load.sum() == float(r.dist_sum.sum())
    for N, d, seed in [(500, 3, 7), (2048, 8, 1)]:
        c = gen.random_regular(N, d, seed)
        rr = oracle.run(c[0], c[1], threads=8, want_load=False)
        if rr.unreachable == 0:
            assert np.all(rr.dist_sum >= s_min(N, d))


def test_bound_formulas(oracle):
    """Sec. 5.3 (time = max load), Eq. (lb) summed over sources, Sec. 2.2 throughput."""
    csr = gen.imase_itoh(64, 4)
    r = oracle.run(csr[0], csr[1])
    E = len(csr[1]); N = 64
    sd = int(r.dist_sum.sum())
    m, b = 2.0 ** 20, 3.125e9
    out = oracle.bound(csr[0], r.load, sd, m, b)
    lmax = float(r.load.max())
    assert out["max_load"] == lmax and out["argmax_arc"] == int(np.argmax(r.load))
    assert out["min_load"] == float(r.load.min())
    assert out["t_sched"] == pytest.approx(lmax * m / b, rel=1e-15)
    assert out["t_lb_nd"] == pytest.approx(sd * m / (N * 4 * b), rel=1e-15)
    assert out["t_lb_links"] == pytest.approx(sd * m / (E * b), rel=1e-15)
    assert out["ratio"] == pytest.approx(lmax * N * 4 / sd, rel=1e-14)
    assert out["throughput"] == pytest.approx((N - 1) * b / lmax, rel=1e-14)
    assert out["t_sched"] >= out["t_lb_links"] >= out["t_lb_nd"]
