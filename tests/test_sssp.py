"""Single-path baseline "SSSP" (Sec. 5.2): shortest paths computed iteration by iteration through a graph whose
link weights reflect the congestion that earlier iterations caused.  The paper gives no weights and does not say
what an iteration is: the reading (weight = commodities routed over the link so far, hop count first, ties to
the lowest link id, an iteration = a block of consecutive sources) is this build's, so parity with the paper is
UNPINNED; what is pinned is that the oracle implements that reading: path enumeration on tiny graphs, a
hand-worked case where the weights decide, and the invariants any single-path shortest-path routing obeys.
GPU: a2a_sssp_loads against the oracle, bit for bit (whole numbers)."""
import numpy as np
import pytest

import a2a_inputs as gen
from helpers import tiny_graphs, paper_values, frac


# ---------------------------------------------------------------------------------------------------------
# CPU: the oracle
# ---------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name", sorted(tiny_graphs()))
@pytest.mark.parametrize("iter_sources", [1, 2, 5, 64])
def test_against_path_enumeration(oracle, name, iter_sources):
    """Every shortest link sequence of every pair written out; the one of least weight taken, ties decided
    from the last link backwards."""
    from oracle import brute_force
    rp, col = tiny_graphs()[name]
    want, chosen = brute_force.sssp(rp, col, iter_sources)
    load, dsum, unr = oracle.sssp(rp, col, iter_sources=iter_sources)
    assert load.tolist() == want
    D = brute_force.distances_by_relaxation([int(x) for x in rp], [int(x) for x in col])
    assert int(dsum.sum()) == sum(d for row in D for d in row if d > 0)
    assert unr == sum(1 for i, row in enumerate(D) for j, d in enumerate(row) if d < 0 and i != j)
    # each chosen sequence is a walk from s to t of D(s,t) links
    tails = np.repeat(np.arange(len(rp) - 1), np.diff(rp))
    for (s, t), path in chosen.items():
        assert len(path) == D[s][t] and tails[path[0]] == s and col[path[-1]] == t
        assert all(col[a] == tails[b] for a, b in zip(path, path[1:]))


def test_weights_decide_where_the_hop_counts_tie(oracle):
    """Two sources, two relays, one target.  Source by source, the first source's path to the target loads
    relay a's link, so the second source goes through relay b; routed in the same iteration both see empty
    links and both take the lower link id.  (The relays are hosts too: each adds its own one-link path to
    the target.)  Worked by hand:
      source by source: s1: s1->a, s1->b, s1->a->t        loads [1+1, 1, 0, 0, 1, 0]
                        s2: a->t now weighs 1, b->t 0      s2->a, s2->b, s2->b->t: [2, 1, 1, 2, 1, 1]
                        a, b: a->t, b->t                   [2, 1, 1, 2, 2, 2]
      two per iteration: s1 and s2 both through a          [2, 1, 2, 1, 2, 0], then a, b: [2, 1, 2, 1, 3, 1]"""
    #      0:s1->a 1:s1->b   2:s2->a 3:s2->b   4:a->t   5:b->t
    rows = [[2, 3], [2, 3], [4], [4], []]
    rp, col = gen.csr_from_rows(rows)
    one, _, _ = oracle.sssp(rp, col, iter_sources=1)
    assert one.tolist() == [2, 1, 1, 2, 2, 2]
    both, _, _ = oracle.sssp(rp, col, iter_sources=2)
    assert both.tolist() == [2, 1, 2, 1, 3, 1]


@pytest.mark.parametrize("make", [lambda: gen.torus([3, 3, 3]), lambda: gen.torus([4, 5]), lambda: gen.hypercube(5),
                                  lambda: gen.random_regular(90, 3, 7), lambda: gen.imase_itoh(81, 8),
                                  lambda: gen.remove_arcs(gen.torus([3, 3, 3]), [3, 50, 101])])
@pytest.mark.parametrize("iter_sources", [1, 7, 64])
def test_single_path_invariants(oracle, make, iter_sources):
    """One path of D(s,t) links per pair: the loads add up to the sum of distances; from one source alone the
    paths form a tree (every other reachable node keeps exactly one path that ends there: inflow - outflow = 1);
    no routing beats the capacity bound sum D / E."""
    rp, col = make()
    N, E = len(rp) - 1, len(col)
    ref = oracle.run(rp, col, want_dist=True)
    load, dsum, unr = oracle.sssp(rp, col, iter_sources=iter_sources)
    assert np.array_equal(dsum, ref.dist_sum) and unr == ref.unreachable
    assert int(load.sum()) == int(ref.dist_sum.sum())
    assert load.max() * E >= ref.dist_sum.sum()
    tails = np.repeat(np.arange(N), np.diff(rp))
    for s in (0, N // 2, N - 1):
        one, _, _ = oracle.sssp(rp, col, s, 1, iter_sources=1)
        used = one > 0
        assert np.all(ref.dist[s][col[used]] == ref.dist[s][tails[used]] + 1)  # only links of shortest paths
        net = np.bincount(col, weights=one, minlength=N) - np.bincount(tails, weights=one, minlength=N)
        reach = ref.dist[s] > 0
        assert np.all(net[reach] == 1) and net[s] == -reach.sum()
        assert np.bincount(col[used], minlength=N)[reach].tolist() == [1] * int(reach.sum())  # one in-link each


def test_first_iteration_is_the_lowest_link_tree(oracle):
    """With every source in one iteration all weights are zero and only the tie rule acts: each node is reached
    over the lowest-numbered link from the level before.  Rebuilt here from the distance matrix alone."""
    rp, col = gen.random_regular(120, 4, 3)
    N, E = len(rp) - 1, len(col)
    dist = oracle.run(rp, col, want_dist=True).dist
    tails = np.repeat(np.arange(N), np.diff(rp))
    want = np.zeros(E, dtype=np.int64)
    for s in range(N):
        parent = np.full(N, -1)
        for a in range(E - 1, -1, -1):  # descending, so the lowest id is written last
            if dist[s][col[a]] == dist[s][tails[a]] + 1 and dist[s][tails[a]] >= 0:
                parent[col[a]] = a
        for t in range(N):
            v = t
            while v != s and parent[v] >= 0:
                want[parent[v]] += 1
                v = tails[parent[v]]
    load, _, _ = oracle.sssp(rp, col, iter_sources=128)
    assert np.array_equal(load, want)


def test_unique_shortest_paths_leave_no_choice(oracle):
    """Imase-Itoh graphs with N = d^k have exactly one shortest path per pair: the single-path loads are the
    EwSP loads, whatever the iteration size."""
    rp, col = gen.imase_itoh(256, 4)
    ewsp = oracle.run(rp, col)
    for k in (1, 64, 256):
        load, _, _ = oracle.sssp(rp, col, iter_sources=k)
        assert np.array_equal(load.astype(np.float64), ewsp.load)


def test_testbed_torus_cannot_beat_the_optimal_flow(oracle):
    """3x3x3 torus: the optimal concurrent flow is f = 1/9 (Sec. 5.1), so every routing has a link of load >= 9;
    the paper finds SSSP clearly worse than the optimum there (Sec. 5.2)."""
    f = frac(paper_values()["torus333_flow_value"])
    rp, col = gen.torus([3, 3, 3])
    for k in (1, 27):
        load, _, _ = oracle.sssp(rp, col, iter_sources=k)
        assert load.max() >= 1 / f
        assert int(load.sum()) == 1458


def test_bad_arguments(oracle):
    rp, col = gen.torus([3, 3])
    with pytest.raises(ValueError):
        oracle.sssp(rp, col, iter_sources=0)
    with pytest.raises(ValueError):
        oracle.sssp(rp, col, 5, 9)


# ---------------------------------------------------------------------------------------------------------
# GPU: a2a_sssp_loads against the oracle
# ---------------------------------------------------------------------------------------------------------

def run_sssp_gpu(topo, s0=0, cnt=None, iter_sources=64, extra_ws=0):
    import torch
    import paper_2309_13541_amd as a2a
    cnt = topo.N - s0 if cnt is None else cnt
    ws_bytes = topo.workspace_bytes(min(iter_sources, (topo.N + 63) // 64 * 64), a2a.WS_SSSP) + extra_ws
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    load = torch.full((max(topo.E, 1),), -7.0, dtype=torch.float64, device="cuda")
    dsum = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    flags = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    topo.sssp_loads(s0, cnt, iter_sources, load=load, dist_sum_total=dsum, flags=flags, workspace=ws)
    torch.cuda.synchronize()
    return load[:topo.E].cpu().numpy(), int(dsum.item()), int(flags.item())


def _gpu_cases():
    from test_gpu_parity import SMALL
    cases = [(n, SMALL[n]) for n in sorted(SMALL) if len(SMALL[n][1])]
    cases += [("C1", gen.named_config("C1")), ("C2", gen.named_config("C2")), ("C3", gen.named_config("C3"))]
    return cases


@pytest.mark.gpu
@pytest.mark.parametrize("case", _gpu_cases(), ids=lambda c: c[0])
def test_gpu_sssp_loads_match_oracle(oracle, case):
    import paper_2309_13541_amd as a2a
    name, (rp, col) = case
    topo = a2a.Topology(rp, col)
    print(f"case {name} N={topo.N} E={topo.E}", flush=True)
    for k in (64, 192):
        want, dsum, unr = oracle.sssp(rp, col, iter_sources=k)
        load, got_sum, flags = run_sssp_gpu(topo, iter_sources=k)
        assert np.array_equal(load, want.astype(np.float64)), k
        assert got_sum == int(dsum.sum()) and flags == (a2a.FLAG_UNREACHABLE if unr else 0)
    topo.close()


@pytest.mark.gpu
def test_gpu_sssp_config_size_ranges_and_arguments(oracle):
    """C4 over all sources (unique shortest paths: also the EwSP loads), a C5 source range at full graph size,
    partial ranges that start inside a batch, a workspace larger than needed, bad arguments."""
    import torch
    import paper_2309_13541_amd as a2a
    rp, col = gen.named_config("C4")
    topo = a2a.Topology(rp, col)
    print("case C4 all sources, 512 per iteration", flush=True)
    want, dsum, _ = oracle.sssp(rp, col, iter_sources=512)
    load, got_sum, flags = run_sssp_gpu(topo, iter_sources=512)
    assert np.array_equal(load, want.astype(np.float64)) and got_sum == int(dsum.sum()) and flags == 0
    assert np.array_equal(load, oracle.run(rp, col, threads=16).load)
    b, st = topo.schedule_bound(torch.from_numpy(load).cuda(), got_sum, flags)
    assert st == 0 and b.max_load == want.max() and b.argmax_arc == int(np.argmax(want))
    topo.close()
    rp, col = gen.named_config("C5")
    topo = a2a.Topology(rp, col)
    print("case C5 sources 30000+1000, 128 per iteration", flush=True)
    want, dsum, _ = oracle.sssp(rp, col, 30000, 1000, iter_sources=128)
    load, got_sum, flags = run_sssp_gpu(topo, 30000, 1000, iter_sources=128, extra_ws=4096)
    assert np.array_equal(load, want.astype(np.float64)) and got_sum == int(dsum.sum()) and flags == 0
    topo.close()
    rp, col = gen.random_regular(500, 5, 17)
    topo = a2a.Topology(rp, col)
    for s0, cnt in ((3, 64), (70, 300), (499, 1), (0, 0)):
        want, dsum, _ = oracle.sssp(rp, col, s0, cnt, iter_sources=64)
        load, got_sum, flags = run_sssp_gpu(topo, s0, cnt)
        assert np.array_equal(load, want.astype(np.float64)) and got_sum == int(dsum.sum())
    ws = torch.empty(topo.workspace_bytes(64, a2a.WS_SSSP), dtype=torch.uint8, device="cuda")
    load = torch.zeros(topo.E, dtype=torch.float64, device="cuda")
    for bad in (0, 63, 100, -64):
        with pytest.raises(a2a.A2AError) as e:
            topo.sssp_loads(0, 500, bad, load=load, workspace=ws)
        assert e.value.status == a2a.ERR_INVALID_ARG
    with pytest.raises(a2a.A2AError) as e:  # the workspace holds one batch, the iteration needs two
        topo.sssp_loads(0, 500, 128, load=load, workspace=ws)
    assert e.value.status == a2a.ERR_WORKSPACE_TOO_SMALL
    topo.close()
