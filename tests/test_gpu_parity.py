"""HIP path vs CPU oracle through the C ABI, element by element (needs an MI355X)."""
import json
import os

import numpy as np
import pytest

import a2a_inputs as gen
from helpers import tiny_graphs, GOLDEN
from gpu_helpers import run_link_loads, run_distances, assert_loads_close, assert_sigma_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def a2a():
    import torch
    assert torch.cuda.is_available()
    import paper_2309_13541_amd as lib
    lib.load_library()
    return lib


def layered_collisions(B=8):
    """64 sources -> 40 nodes (A) -> B nodes -> 1..B leaves each, plus filler nodes with a link into
    the sources.  Level 1 holds A with all 64 sources per node, level 2 is sparse on average but every
    node of A has B successors there for every source: the backward pass of level 1 adds B different
    coef values per (node, source), which is where the order of additions could show.  With B = 12 the
    nodes of A have more than eight out-links (a second tile of links into the same accumulators)."""
    S, A = 64, 40
    a0, b0 = S, S + A
    c0 = b0 + B
    leaves = sum(range(1, B + 1))
    N = c0 + leaves + 52
    rows = [[a0 + (s + 3 * i) % A for i in range(A)] for s in range(S)]
    rows += [[b0 + (a + i) % B for i in range(B)] for a in range(A)]
    nxt = c0
    for b in range(B):
        rows.append(list(range(nxt, nxt + b + 1)))
        nxt += b + 1
    rows += [[] for _ in range(leaves)]
    rows += [[i % S] for i in range(52)]
    assert len(rows) == N
    return gen.csr_from_rows(rows)


def dense_layers(K=7, W=64, seed=77):
    """K layers of W nodes in a cycle, every node linked to about 9 in 10 nodes of the next layer.  Every level
    from 1 to K is well filled (64/K sources per node) and the largest in-degree is 63: the forward launches of
    levels 2..5 may read the level before in single precision (path counts on level 4 are below 63^4 < 2^24),
    those of levels 6..K must not (the counts there go past 2^24, up to about 58^6)."""
    rng = np.random.default_rng(seed)
    rows = []
    for k in range(K):
        nxt = ((k + 1) % K) * W
        for _ in range(W):
            keep = rng.random(W) < 0.9
            keep[rng.integers(W)] = True
            rows.append([nxt + int(j) for j in np.nonzero(keep)[0]])
    return gen.csr_from_rows(rows)


def funnel_layers(widths, seed):
    """Nodes 0..63 (the sources the tests run it with) -> 4 merge nodes (16 sources each) -> 4 hubs -> layers
    of the given widths; hub h reaches 70 % of the first layer (a different window each), a node of a later
    layer has 9..16 in-links from the layer before.  For those 64 sources, level l >= 3 is layer l - 3 (all its
    nodes from the second layer on, with almost all sources each): the widths choose how full each level is,
    hence which kernel flavour runs it, and the largest in-degree, 16, fixes from where on path counts are kept
    in double precision (level 6: 16^6 = 2^24).  The four groups of sources see different counts."""
    rng = np.random.default_rng(seed)
    first = 64 + 4 + 4
    starts = [first]
    for w in widths:
        starts.append(starts[-1] + w)
    rows = [[64 + s // 16] for s in range(64)]
    rows += [[68 + h] for h in range(4)]
    w0 = widths[0]
    span = max(1, (7 * w0) // 10)
    rows += [[first + (h * (w0 - span) // 3 + i) % w0 for i in range(span)] for h in range(4)]
    rows += [[] for _ in range(starts[-1] - first)]
    for k in range(1, len(widths)):
        wp = widths[k - 1]
        for j in range(widths[k]):
            deg = min(wp, int(rng.integers(9, 17)))
            for u in rng.choice(wp, size=deg, replace=False):
                rows[starts[k - 1] + int(u)].append(starts[k] + j)
    return gen.csr_from_rows([sorted(r) for r in rows])


# level:            3    4    5    6    7    8    9   10
FUNNELS = {
    "funnel_a": ([100, 100, 30, 100, 100, 4, 100, 30], 5),   # level 6: dense after sparse
    "funnel_b": ([100, 100, 100, 100, 30, 100, 4, 100], 6),  # level 6: dense after dense
    "funnel_c": ([100, 100, 100, 30, 100, 100, 30, 100], 7),  # level 6: a few sources per node
    "funnel_d": ([100, 100, 100, 4, 100, 100, 100, 30], 8),   # level 6: under two sources per node
}


SMALL = dict(tiny_graphs())
SMALL.update({
    "torus3x3x3": gen.torus([3, 3, 3]),
    "ring_odd_131": gen.ring(131),              # diameter 130, N not a multiple of 64
    "biring_200": gen.bidirectional_ring(200),  # diameter 100 = N/2
    # the distance output builds 3, 5 or 7 bit planes (deepest level below 8, 32, 128), one source at a time up to
    # 255, through an LDS tile beyond: both sides of every limit
    "ring_8": gen.ring(8),
    "ring_9": gen.ring(9),
    "ring_32": gen.ring(32),
    "ring_33": gen.ring(33),
    "ring_128": gen.ring(128),
    "ring_129": gen.ring(129),
    "ring_255": gen.ring(255),                  # diameter 254
    "ring_256": gen.ring(256),                  # diameter 255: deepest that the bit-plane distance output takes
    "ring_300": gen.ring(300),
    "kautz_81_8": gen.imase_itoh(81, 8),
    "kautz_100_3": gen.imase_itoh(100, 3),
    "rr_300_4": gen.random_regular(300, 4, 5),
    "rr_257_8": gen.random_regular(257, 8, 11),
    "torus_5x13": gen.torus([5, 13]),           # N = 65: one node into the second batch
    "hub_in_100": gen.csr_from_rows([[99] for _ in range(99)] + [list(range(99))]),  # degree 99
    "punctured_333": gen.remove_arcs(gen.torus([3, 3, 3]), [3, 50, 101]),
    "punctured_nodes_333": gen.remove_nodes(gen.torus([3, 3, 3]), [0, 13, 20]),
    "two_components": gen.csr_from_rows([[1], [0], [3], [4], [2]]),
    "no_links": gen.csr_from_rows([[], [], []]),
    "chain_2pow54": gen.csr_from_rows([[i + 1, i + 1] for i in range(54)] + [[]]),
    # path counts from node 0 are tiny, from node 1 they reach 2^30
    "late_blowup": gen.csr_from_rows([[]] + [[i + 1, i + 1] for i in range(1, 31)] + [[]]),
    "layered_collisions": layered_collisions(),
    "layered_collisions_wide": layered_collisions(12),
    "dense_layers": dense_layers(),
})


@pytest.mark.parametrize("name", sorted(SMALL))
def test_small_graphs_everything(a2a, oracle, name):
    rp, col = SMALL[name]
    print(f"case {name} N={len(rp) - 1} E={len(col)}", flush=True)
    o = oracle.run(rp, col, want_dist=True, want_sigma=True)
    topo = a2a.Topology(rp, col)
    dist, sigma, dsum, unr, flags = run_distances(topo)
    assert np.array_equal(dist, o.dist)
    assert np.array_equal(dsum, o.dist_sum)
    assert unr == o.unreachable
    assert flags == o.flags
    if not (o.flags & 1):
        assert_sigma_equal(sigma, o.sigma)
    else:  # counts beyond 2^53 are flagged, and still agree to fp64 rounding
        np.testing.assert_allclose(sigma, o.sigma.astype(np.float64), rtol=1e-15)
    load, dtot, lflags = run_link_loads(topo)
    assert dtot == int(o.dist_sum.sum()) and lflags == o.flags
    if len(col):
        assert_loads_close(load, o.load)
    topo.close()


def random_digraph(seed):
    """A seeded digraph of no particular shape: 1 to 330 nodes, out-degrees from 0 to 12 drawn per node (so
    in-degrees vary as well, some nodes have none), parallel links left in, self-loops dropped; one in four
    graphs gets a few nodes without any links."""
    rng = np.random.default_rng(seed)
    N = int(rng.integers(1, 331))
    dmax = int(rng.integers(1, 13))
    rows = []
    for u in range(N):
        deg = int(rng.integers(1 if seed % 2 else 0, dmax + 1))  # odd seeds: every node has an out-link
        rows.append([int(w) for w in rng.integers(0, N, size=deg) if int(w) != u])
    if seed % 4 == 0:
        for u in rng.integers(0, N, size=min(N, 5)):
            rows[int(u)] = []
    return gen.csr_from_rows(rows)


@pytest.mark.parametrize("block", range(8))
def test_random_digraphs_everything(a2a, oracle, block):
    """160 seeded random digraphs (20 per case): distances, path counts, sums, flags and link loads against the
    oracle, all sources and one partial source range each."""
    for seed in range(20 * block, 20 * block + 20):
        rp, col = random_digraph(seed)
        N = len(rp) - 1
        print(f"seed {seed} N={N} E={len(col)}", flush=True)
        o = oracle.run(rp, col, want_dist=True, want_sigma=True)
        topo = a2a.Topology(rp, col)
        dist, sigma, dsum, unr, flags = run_distances(topo)
        assert np.array_equal(dist, o.dist) and np.array_equal(dsum, o.dist_sum), seed
        assert unr == o.unreachable and flags == o.flags, seed
        if not (o.flags & 1):
            assert_sigma_equal(sigma, o.sigma)
        load, dtot, lflags = run_link_loads(topo)
        assert dtot == int(o.dist_sum.sum()) and lflags == o.flags, seed
        if len(col):
            assert_loads_close(load, o.load)
            s0 = seed % N
            cnt = min(N - s0, 1 + seed % 97)
            part = oracle.run(rp, col, s0, cnt)
            pl, pd, pf = run_link_loads(topo, s0, cnt)
            assert pd == int(part.dist_sum.sum()), seed
            assert_loads_close(pl, part.load)
        topo.close()


@pytest.mark.parametrize("name", sorted(FUNNELS))
def test_funnels_precision_boundary(a2a, oracle, name):
    """Graphs whose levels 3..10 (for sources 0..63) are as full as chosen, with the change from single- to
    double-precision path counts at level 6: every kernel flavour on either side of it and across it."""
    rp, col = funnel_layers(*FUNNELS[name])
    print(f"case {name} N={len(rp) - 1} E={len(col)}", flush=True)
    o = oracle.run(rp, col, 0, 64, want_dist=True, want_sigma=True)
    assert not (o.flags & 1)
    topo = a2a.Topology(rp, col)
    dist, sigma, dsum, unr, flags = run_distances(topo, 0, 64)
    assert np.array_equal(dist, o.dist) and np.array_equal(dsum, o.dist_sum)
    assert unr == o.unreachable and flags == o.flags
    assert_sigma_equal(sigma, o.sigma)
    load, dtot, lflags = run_link_loads(topo, 0, 64)
    assert dtot == int(o.dist_sum.sum()) and lflags == o.flags
    assert_loads_close(load, o.load)
    topo.close()


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_configs_loads_and_sums(a2a, oracle, name):
    rp, col = gen.named_config(name)
    print(f"case {name}", flush=True)
    o = oracle.run(rp, col, threads=16)
    topo = a2a.Topology(rp, col)
    load, dtot, flags = run_link_loads(topo)
    assert dtot == int(o.dist_sum.sum()) and flags == 0
    assert_loads_close(load, o.load)
    if name == "C4":  # unique shortest paths: whole-number loads, exact on both sides
        assert np.array_equal(load, o.load)
    # schedule figures against the oracle's formulas
    b, st = topo.schedule_bound(topo_load_tensor(load), dtot, flags, 2.0 ** 20, 3.125e9)
    ob = oracle.bound(rp, load, dtot, 2.0 ** 20, 3.125e9)  # same load vector on both sides
    assert st == 0
    for k in ("max_load", "min_load", "t_sched", "t_lb_nd", "t_lb_links", "ratio", "throughput",
              "flow_value", "throughput_upper"):
        assert getattr(b, k) == pytest.approx(ob[k], rel=1e-14), k
    assert b.argmax_arc == ob["argmax_arc"]
    assert b.n_links == len(col) and b.n_nodes == len(rp) - 1 and b.sum_dist == dtot
    topo.close()


def topo_load_tensor(load_np):
    import torch
    return torch.from_numpy(np.ascontiguousarray(load_np)).cuda()


@pytest.mark.parametrize("name,ranges", [
    ("C1", [(0, 64)]),
    ("C2", [(0, 1024)]),
    ("C3", [(0, 300), (4000, 96)]),
    ("C4", [(0, 130), (9000, 64), (16384 - 70, 70)]),
    ("C5", [(0, 64), (30000, 100), (65536 - 65, 65)]),
])
def test_configs_distances_and_sigma(a2a, oracle, name, ranges):
    rp, col = gen.named_config(name)
    topo = a2a.Topology(rp, col)
    for s0, cnt in ranges:
        print(f"case {name} sources {s0}+{cnt}", flush=True)
        o = oracle.run(rp, col, s0, cnt, threads=16, want_dist=True, want_sigma=True, want_load=False)
        dist, sigma, dsum, unr, flags = run_distances(topo, s0, cnt)
        assert np.array_equal(dist, o.dist)
        assert_sigma_equal(sigma, o.sigma)
        assert np.array_equal(dsum, o.dist_sum)
        assert unr == 0 and flags == 0
        # distances alone (no path counting) take another code path
        dist2, _, dsum2, _, _ = run_distances(topo, s0, cnt, want_sigma=False)
        assert np.array_equal(dist2, o.dist) and np.array_equal(dsum2, o.dist_sum)
    topo.close()


def test_c5_source_ranges_loads(a2a, oracle):
    """Loads of sub-ranges of sources at full C5 size, element by element."""
    rp, col = gen.named_config("C5")
    topo = a2a.Topology(rp, col)
    for s0, cnt in [(0, 512), (41000, 200), (65536 - 100, 100)]:
        print(f"case C5 sources {s0}+{cnt}", flush=True)
        o = oracle.run(rp, col, s0, cnt, threads=16)
        load, dtot, flags = run_link_loads(topo, s0, cnt)
        assert dtot == int(o.dist_sum.sum()) and flags == 0
        assert_loads_close(load, o.load)
    topo.close()


@pytest.fixture(scope="module")
def c5_full(a2a):
    """One full C5 run in the benchmark's launch configuration (recommended workspace, all 1024 batches in
    one group), shared by the tests below."""
    rp, col = gen.named_config("C5")
    topo = a2a.Topology(rp, col)
    print("case C5 full", flush=True)
    load, dtot, flags = run_link_loads(topo)
    yield rp, col, topo, load, dtot, flags
    topo.close()


def test_c5_full_loads_element_by_element(c5_full, oracle):
    """All 524 283 link loads of the full 65 536-source run against a live oracle run, link by link."""
    rp, col, topo, load, dtot, flags = c5_full
    o = oracle.run(rp, col, threads=16)
    assert flags == o.flags == 0 and o.unreachable == 0
    assert dtot == int(o.dist_sum.sum())
    assert_loads_close(load, o.load)
    assert int(np.argmax(load)) == int(np.argmax(o.load))


def test_c5_full_against_stored_oracle_values(c5_full, oracle):
    """The same run against the stored oracle figures (sum of distances, extrema, 257 sampled links) and
    the load-sum invariant."""
    with open(os.path.join(GOLDEN, "oracle_config_values.json")) as f:
        g = json.load(f)["C5"]
    rp, col, topo, load, dtot, flags = c5_full
    assert dtot == g["sum_dist"] and flags == 0
    want = np.array([float.fromhex(x) for x in g["sample_loads"]])
    assert_loads_close(load[np.asarray(g["sample_ids"])], want)
    assert float(load.max()) == pytest.approx(float.fromhex(g["max_load"]), rel=1e-9)
    assert float(load.min()) == pytest.approx(float.fromhex(g["min_load"]), rel=1e-9)
    assert int(np.argmax(load)) == g["argmax_arc"]
    assert float(load.sum()) == pytest.approx(float(dtot), rel=1e-10)
    b, st = topo.schedule_bound(topo_load_tensor(load), dtot, flags)
    assert st == 0 and b.argmax_arc == g["argmax_arc"]
    assert b.max_load * b.n_links / dtot == pytest.approx(g["ratio_links"], rel=1e-9)


def test_c5_full_distance_matrix_bit_exact(a2a, oracle):
    """a2a_distances over all 65 536 sources in one call (the configuration the benchmark times): the whole
    int32 matrix and the per-source sums against the oracle, 2048 rows at a time."""
    import torch
    rp, col = gen.named_config("C5")
    topo = a2a.Topology(rp, col)
    N = topo.N
    print("case C5 full distance matrix", flush=True)
    ws = topo.alloc_workspace(N, a2a.WS_DISTANCES)
    dist = torch.full((N, N), -9, dtype=torch.int32, device="cuda")
    dsum = torch.full((N,), -1, dtype=torch.int64, device="cuda")
    unr = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    topo.distances(0, N, dist=dist, dist_sum=dsum, unreachable=unr, workspace=ws)
    torch.cuda.synchronize()
    assert int(unr.item()) == 0
    got_sum = dsum.cpu().numpy()
    chunk = 2048
    for s0 in range(0, N, chunk):
        o = oracle.run(rp, col, s0, chunk, threads=16, want_dist=True, want_load=False)
        assert np.array_equal(dist[s0:s0 + chunk].cpu().numpy(), o.dist), s0
        assert np.array_equal(got_sum[s0:s0 + chunk], o.dist_sum), s0
        if s0 % (8 * chunk) == 0:
            print(f"  rows {s0}..{s0 + chunk - 1} ok", flush=True)
    del dist, ws
    # path counts on 4096 sources spread over the range (the with-sigma code path), 512 at a time
    for s0 in range(100, N, N // 8):
        o = oracle.run(rp, col, s0, 512, threads=16, want_dist=True, want_sigma=True, want_load=False)
        d2, sg, ds2, u2, f2 = run_distances(topo, s0, 512)
        assert np.array_equal(d2, o.dist) and np.array_equal(ds2, o.dist_sum)
        assert_sigma_equal(sg, o.sigma)
        assert u2 == 0 and f2 == 0
    topo.close()


def test_workspace_size_and_reruns(a2a, oracle):
    """One batch at a time vs several vs all batches together, and the same workspace twice: the same bits
    every time (every batch picks its lane layouts from its own level sizes, every sum has a fixed order)."""
    rp, col = gen.random_regular(1000, 6, 21)
    topo = a2a.Topology(rp, col)
    full = run_link_loads(topo)
    least = topo.workspace_bytes(topo.N, a2a.WS_LOADS | a2a.WS_MINIMAL)
    one = run_link_loads(topo, max_ws=least)
    three = run_link_loads(topo, max_ws=3 * least)
    assert np.array_equal(one[0], full[0])
    assert np.array_equal(three[0], full[0])
    assert full[1:] == one[1:] == three[1:]
    for ws in (None, least, 3 * least):  # run-to-run bitwise determinism
        a = run_link_loads(topo, max_ws=ws)
        b = run_link_loads(topo, max_ws=ws)
        assert np.array_equal(a[0], b[0])
    # the same where eight or twelve different values are added per (node, source)
    for name in ("layered_collisions", "layered_collisions_wide"):
        rp2, col2 = SMALL[name]
        topo2 = a2a.Topology(rp2, col2)
        first = run_link_loads(topo2, 0, 64)  # the 64 designed sources alone: one batch, levels as described
        assert_loads_close(first[0], oracle.run(rp2, col2, 0, 64).load)
        for _ in range(3):
            assert np.array_equal(run_link_loads(topo2, 0, 64)[0], first[0])
        topo2.close()
    d_full = run_distances(topo)
    d_one = run_distances(topo, max_ws=topo.workspace_bytes(topo.N, a2a.WS_SIGMA | a2a.WS_MINIMAL))
    for x, y in zip(d_full[:3], d_one[:3]):
        assert np.array_equal(x, y)
    topo.close()


def test_empty_and_partial_source_ranges(a2a, oracle):
    rp, col = gen.torus([7, 11])
    topo = a2a.Topology(rp, col)
    load, dtot, flags = run_link_loads(topo, 5, 0)
    assert np.all(load == 0) and dtot == 0 and flags == 0
    for s0, cnt in [(0, 1), (76, 1), (3, 64), (10, 67)]:
        o = oracle.run(rp, col, s0, cnt, want_dist=True, want_sigma=True)
        load, dtot, flags = run_link_loads(topo, s0, cnt)
        assert_loads_close(load, o.load)
        assert dtot == int(o.dist_sum.sum())
        dist, sigma, dsum, unr, fl = run_distances(topo, s0, cnt)
        assert np.array_equal(dist, o.dist) and np.array_equal(dsum, o.dist_sum)
        assert_sigma_equal(sigma, o.sigma)
    topo.close()


def test_error_paths_on_device(a2a):
    import torch
    rp, col = gen.torus([4, 4])
    topo = a2a.Topology(rp, col)
    load = torch.zeros(topo.E, dtype=torch.float64, device="cuda")
    tiny = torch.empty(512, dtype=torch.uint8, device="cuda")
    with pytest.raises(a2a.A2AError) as e:
        topo.link_loads(0, 16, load=load, workspace=tiny)
    assert e.value.status == a2a.ERR_WORKSPACE_TOO_SMALL
    ws = topo.alloc_workspace(16, a2a.WS_LOADS)
    with pytest.raises(a2a.A2AError) as e:
        topo.link_loads(10, 7, load=load, workspace=ws)
    assert e.value.status == a2a.ERR_INVALID_ARG
    # disconnected topology: loads are still produced, schedule_bound reports it
    t2 = a2a.Topology(*gen.csr_from_rows([[1], [0], [3], [4], [2]]))
    l2, d2, f2 = run_link_loads(t2)
    assert f2 & a2a.FLAG_UNREACHABLE
    b, st = t2.schedule_bound(topo_load_tensor(l2), d2, f2, allow_disconnected=True)
    assert st == a2a.ERR_DISCONNECTED and b.max_load == 3.0
    topo.close(); t2.close()


def test_kautz_approaches_the_tree_bound(a2a, oracle):
    """Sec. 5.4: generalized Kautz graphs come close to the lower bound of Theorem 1, the ratio
    approaching 1 for large N; a 2D torus of the same degree falls behind as N grows.  Distance
    sums from the device (no dist matrix, no path counts), bound from a2a_tree_lower_bound."""
    import torch

    def ratio(csr, d):
        rp, col = csr
        topo = a2a.Topology(rp, col)
        N = topo.N
        ws = topo.alloc_workspace(N, a2a.WS_DISTANCES)
        dsum = torch.zeros(N, dtype=torch.int64, device="cuda")
        unr = torch.zeros(1, dtype=torch.int64, device="cuda")
        topo.distances(0, N, dist_sum=dsum, unreachable=unr, workspace=ws)
        torch.cuda.synchronize()
        got = dsum.cpu().numpy()
        o = oracle.run(rp, col, threads=16, want_load=False)
        assert np.array_equal(got, o.dist_sum) and int(unr.item()) == 0
        smin = a2a.tree_lower_bound(N, d).s_min
        assert smin == oracle.tree_sum(N, d)
        assert got.min() >= smin  # every source obeys the bound
        topo.close()
        return float(got.sum()) / (N * smin)

    kautz = {N: ratio(gen.imase_itoh(N, 4), 4) for N in (27, 64, 256, 1024, 4096, 16384)}
    print("sum D / (N * S_min), Imase-Itoh d=4:", kautz, flush=True)
    assert all(r >= 1.0 for r in kautz.values())
    assert kautz[16384] < kautz[4096] < kautz[1024] < kautz[256] < kautz[64] < 1.01
    assert kautz[16384] < 1.004
    torus = {k * k: ratio(gen.torus([k, k]), 4) for k in (8, 16, 32)}
    print("2D torus:", torus, flush=True)
    assert torus[64] < torus[256] < torus[1024] and torus[1024] > 3.0


def test_disabled_links_and_hosts(a2a, oracle):
    """Degree-irregular topologies made by disabling random links (Sec. 5.3, the N=81, d=8
    generalized Kautz experiment) and by puncturing a torus (Sec. 5.2): parity with the oracle,
    and a disconnected outcome is reported, not hidden."""
    rng = np.random.default_rng(20230913)
    base = gen.imase_itoh(81, 8)
    E = len(base[1])
    for n_off in (3, 20, 80, 200):
        rp, col = gen.remove_arcs(base, rng.choice(E, size=n_off, replace=False))
        print(f"case kautz_81_8 minus {n_off} links", flush=True)
        o = oracle.run(rp, col, want_dist=True, want_sigma=True)
        topo = a2a.Topology(rp, col)
        dist, sigma, dsum, unr, flags = run_distances(topo)
        assert np.array_equal(dist, o.dist) and np.array_equal(dsum, o.dist_sum)
        assert_sigma_equal(sigma, o.sigma)
        assert unr == o.unreachable and flags == o.flags
        load, dtot, lflags = run_link_loads(topo)
        assert_loads_close(load, o.load)
        b, st = topo.schedule_bound(topo_load_tensor(load), dtot, lflags, allow_disconnected=True)
        assert (st == a2a.ERR_DISCONNECTED) == (o.unreachable > 0)
        ob = oracle.bound(rp, o.load, int(o.dist_sum.sum()))
        assert b.max_load == pytest.approx(ob["max_load"], rel=1e-9)
        if o.unreachable == 0:  # the capacity bound with the true link count still holds
            assert b.t_sched >= b.t_lb_links * (1 - 1e-12)
        topo.close()
    torus = gen.torus([3, 3, 3])
    for kind in ("links", "hosts"):
        for trial in range(3):
            if kind == "links":
                csr = gen.remove_arcs(torus, rng.choice(162, size=3, replace=False))
            else:
                csr = gen.remove_nodes(torus, rng.choice(27, size=3, replace=False))
            o = oracle.run(*csr)
            topo = a2a.Topology(*csr)
            load, dtot, lflags = run_link_loads(topo)
            assert dtot == int(o.dist_sum.sum()) and lflags == o.flags
            assert_loads_close(load, o.load)
            topo.close()


LAYOUTS = ("rows", "spread", "node_source", "node_link")


def _flavours(a2a, rp, col, src_count=None):
    """Which lane layout each batch picked on each level, with the precision of the path counts it read and
    wrote (f = single, d = double): the library's profile reports them from the batches' own level sizes."""
    import torch
    topo = a2a.Topology(rp, col)
    cnt = topo.N if src_count is None else src_count
    ws = topo.alloc_workspace(cnt, a2a.WS_LOADS)
    load = torch.empty(max(topo.E, 1), dtype=torch.float64, device="cuda")
    topo.profile_enable(1)
    topo.link_loads(0, cnt, load=load, workspace=ws)
    p = topo.profile_read()
    topo.profile_enable(0)
    seen = set()
    for i, layout in enumerate(LAYOUTS):
        for j, prec in enumerate(("_ff", "_fd", "_dd")):
            if (p["fwd_flavours"] >> (3 * i + j)) & 1:
                seen.add("fwd_" + layout + prec)
        for j, prec in enumerate(("_f", "_d")):
            if (p["bwd_flavours"] >> (2 * i + j)) & 1:
                seen.add("bwd_" + layout + prec)
    topo.close()
    return seen


def test_parity_set_reaches_every_kernel_flavour(a2a):
    """The level kernels come in flavours picked from how full a level is and from the precision the path
    counts of the levels involved are kept in; the graphs of test_small_graphs_everything and
    test_funnels_precision_boundary must between them run every one (else parity says nothing about the ones
    left out)."""
    seen = set()
    for name in sorted(SMALL):
        rp, col = SMALL[name]
        if len(col) == 0:
            continue
        got = _flavours(a2a, rp, col)
        print(name, sorted(got), flush=True)
        seen |= got
    for name in sorted(FUNNELS):
        got = _flavours(a2a, *funnel_layers(*FUNNELS[name]), src_count=64)
        print(name, sorted(got), flush=True)
        seen |= got
    want = {"fwd_" + f + p for f in LAYOUTS for p in ("_ff", "_fd", "_dd")}
    want |= {"bwd_" + f + p for f in LAYOUTS for p in ("_f", "_d")}
    assert want <= seen, sorted(want - seen)
