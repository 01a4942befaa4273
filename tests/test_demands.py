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


# ---------------------------------------------------------------------------------------------------------
# GPU: a2a_link_loads_demand against the oracle
# ---------------------------------------------------------------------------------------------------------

def run_demand_gpu(topo, dem_by_source, src_begin=0, max_ws=None):
    """dem_by_source: numpy [src_count][N] (the oracle's layout); the library takes it by target."""
    import torch
    import paper_2309_13541_amd as a2a
    cnt = dem_by_source.shape[0]
    ws = topo.alloc_workspace(cnt, a2a.WS_LOADS, max_ws)
    dem = torch.from_numpy(np.ascontiguousarray(dem_by_source.T)).cuda()  # [N][src_count]
    load = torch.full((max(topo.E, 1),), -7.0, dtype=torch.float64, device="cuda")
    wd = torch.full((1,), -1.0, dtype=torch.float64, device="cuda")
    dsum = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    flags = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    topo.link_loads_demand(src_begin, cnt, demand=dem, load=load, weighted_dist=wd, dist_sum_total=dsum,
                           flags=flags, workspace=ws)
    torch.cuda.synchronize()
    return load[:topo.E].cpu().numpy(), float(wd.item()), int(dsum.item()), int(flags.item())


def _gpu_cases():
    from test_gpu_parity import SMALL, FUNNELS, funnel_layers
    cases = [(n, SMALL[n], None) for n in sorted(SMALL) if len(SMALL[n][1]) and n not in ("chain_2pow54",)]
    cases += [(n, funnel_layers(*FUNNELS[n]), 64) for n in sorted(FUNNELS)]
    cases += [("C1", gen.named_config("C1"), None), ("C2", gen.named_config("C2"), None)]
    return cases


@pytest.mark.gpu
@pytest.mark.parametrize("case", _gpu_cases(), ids=lambda c: c[0])
def test_gpu_demand_loads_match_oracle(oracle, case):
    """Every kernel flavour with demands (the graphs are those of the flavour test of test_gpu_parity)."""
    import paper_2309_13541_amd as a2a
    from gpu_helpers import assert_loads_close
    name, (rp, col), cnt = case
    N = len(rp) - 1
    cnt = N if cnt is None else cnt
    print(f"case {name} N={N} E={len(col)} sources={cnt}", flush=True)
    dem = seeded_demand(cnt, N, 1000 + N)
    want, want_wd = oracle.run_demand(rp, col, dem)
    ref = oracle.run(rp, col, 0, cnt)
    topo = a2a.Topology(rp, col)
    load, wd, dsum, flags = run_demand_gpu(topo, dem)
    assert_loads_close(load, want)
    assert wd == pytest.approx(want_wd, rel=1e-12)
    assert dsum == int(ref.dist_sum.sum()) and flags == ref.flags
    topo.close()


def big_demand(n_src, N, seed):
    """Whole-number demands 0..7 (one in eight zero) from numpy's seeded generator: an input, drawn once and
    handed to both sides."""
    return np.random.default_rng(seed).integers(0, 8, size=(n_src, N)).astype(np.float64)


def oracle_demand_sliced(oracle, rp, col, dem, src_begin, slices=16):
    """The serial oracle on consecutive slices of the sources, one thread each (the C call releases the
    interpreter lock); loads and weighted distances of the slices added in source order."""
    from concurrent.futures import ThreadPoolExecutor
    cnt = dem.shape[0]
    cuts = [cnt * i // slices for i in range(slices + 1)]
    jobs = [(a, b) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    with ThreadPoolExecutor(max_workers=len(jobs)) as ex:
        parts = list(ex.map(lambda ab: oracle.run_demand(rp, col, dem[ab[0]:ab[1]], src_begin + ab[0]), jobs))
    load = np.zeros(len(col))
    wd = 0.0
    for l, w in parts:
        load += l
        wd += w
    return load, wd


@pytest.mark.gpu
@pytest.mark.parametrize("name,s0,cnt", [("C3", 0, 4096), ("C4", 0, 16384), ("C5", 20000, 640)])
def test_gpu_demand_loads_at_config_size(oracle, name, s0, cnt):
    """Unequal demands at the size of the benchmark configurations, link by link: C3 and C4 over all sources,
    C5 over ten batches of sources."""
    import paper_2309_13541_amd as a2a
    from gpu_helpers import assert_loads_close
    rp, col = gen.named_config(name)
    N = len(rp) - 1
    print(f"case {name} N={N} E={len(col)} sources {s0}+{cnt}", flush=True)
    dem = big_demand(cnt, N, 4000 + N)
    want, want_wd = oracle_demand_sliced(oracle, rp, col, dem, s0)
    topo = a2a.Topology(rp, col)
    load, wd, dsum, flags = run_demand_gpu(topo, dem, s0)
    assert flags == 0
    assert_loads_close(load, want)
    assert wd == pytest.approx(want_wd, rel=1e-12)
    topo.close()


@pytest.mark.gpu
def test_gpu_unit_demand_matrix_gives_the_unit_loads(oracle):
    from gpu_helpers import run_link_loads
    import paper_2309_13541_amd as a2a
    for rp, col in (gen.random_regular(300, 4, 5), gen.torus([5, 13])):
        N = len(rp) - 1
        topo = a2a.Topology(rp, col)
        unit, dsum, _ = run_link_loads(topo)
        load, wd, dsum2, _ = run_demand_gpu(topo, np.ones((N, N)))
        # same sums in the same order, except that the deepest level is visited by the backward kernel
        np.testing.assert_allclose(load, unit, rtol=1e-13)
        assert wd == float(dsum) and dsum2 == dsum
        topo.close()


@pytest.mark.gpu
def test_gpu_demand_source_ranges_groups_and_reruns(oracle):
    import paper_2309_13541_amd as a2a
    from gpu_helpers import assert_loads_close
    rp, col = gen.random_regular(1000, 6, 21)
    N = 1000
    topo = a2a.Topology(rp, col)
    dem = seeded_demand(N, N, 9)
    want, want_wd = oracle.run_demand(rp, col, dem)
    full = run_demand_gpu(topo, dem)
    assert_loads_close(full[0], want)
    assert full[1] == pytest.approx(want_wd, rel=1e-12)
    again = run_demand_gpu(topo, dem)
    assert np.array_equal(full[0], again[0]) and full[1] == again[1]  # run-to-run bitwise
    least = topo.workspace_bytes(N, a2a.WS_LOADS | a2a.WS_MINIMAL)
    small = run_demand_gpu(topo, dem, max_ws=least)  # one super-batch at a time: several groups
    assert np.array_equal(small[0], full[0]) and small[1] == full[1]  # the grouping changes no bit
    # a source range that starts and ends inside a batch
    part, part_wd = oracle.run_demand(rp, col, dem[70:203], 70)
    got = run_demand_gpu(topo, dem[70:203], 70)
    assert_loads_close(got[0], part)
    assert got[1] == pytest.approx(part_wd, rel=1e-12)
    topo.close()


@pytest.mark.gpu
def test_gpu_demand_argument_checks():
    import torch
    import paper_2309_13541_amd as a2a
    rp, col = gen.torus([4, 4])
    topo = a2a.Topology(rp, col)
    ws = topo.alloc_workspace(16, a2a.WS_LOADS)
    load = torch.zeros(topo.E, dtype=torch.float64, device="cuda")
    with pytest.raises(a2a.A2AError) as e:
        topo.link_loads_demand(0, 16, demand=None, load=load, workspace=ws)
    assert e.value.status == a2a.ERR_INVALID_ARG
    # no sources: zero loads and zero weighted distance
    wd = torch.full((1,), 5.0, dtype=torch.float64, device="cuda")
    dem = torch.ones((16, 1), dtype=torch.float64, device="cuda")
    load.fill_(3.0)
    topo.link_loads_demand(4, 0, demand=dem, load=load, weighted_dist=wd, workspace=ws)
    torch.cuda.synchronize()
    assert float(wd.item()) == 0.0 and float(load.abs().sum().item()) == 0.0
    topo.close()
