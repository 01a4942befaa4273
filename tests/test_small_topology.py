"""Topologies too small to fill the chip: 2, 4 or 8 waves share each block of 64 nodes, depending on how many batches
a launch holds.  Link loads against the oracle, and the same bits for every workspace size.  (Needs an MI355X.)"""
import numpy as np
import pytest

import a2a_inputs as gen
from gpu_helpers import run_link_loads, assert_loads_close
from test_gpu_parity import layered_collisions, dense_layers, random_digraph

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def a2a():
    import torch
    assert torch.cuda.is_available()
    import paper_2309_13541_amd as lib
    lib.load_library()
    return lib


def all_group_sizes(a2a, topo, src_begin=0, src_count=None):
    """(load, dist sum, flags) with a workspace for the whole range, after checking that workspaces for one and for
    three batches give the same bits (the fewer batches share a launch, the more waves share a block of nodes)."""
    whole = run_link_loads(topo, src_begin, src_count)
    for batches in (1, 3):
        small = topo.workspace_bytes(64 * batches, a2a.WS_LOADS)
        again = run_link_loads(topo, src_begin, src_count, small)
        assert np.array_equal(again[0], whole[0]) and again[1:] == whole[1:]
    return whole


def small_cases():
    yield "C1", gen.named_config("C1")
    yield "C2", gen.named_config("C2")
    yield "ring 300 (299 levels)", gen.ring(300)
    yield "bidirectional ring 257", gen.bidirectional_ring(257)
    yield "torus 12x11", gen.torus([12, 11])
    yield "random 5-regular 1500", gen.random_regular(1500, 5, 3)
    yield "Imase-Itoh 1000, 3", gen.imase_itoh(1000, 3)
    yield "complete bipartite 40", gen.complete_bipartite(40)
    yield "layered collisions 8", layered_collisions(8)
    yield "layered collisions 12", layered_collisions(12)
    yield "dense layers (double-precision levels)", dense_layers()
    yield "hypercube 11", gen.hypercube(11)
    yield "two nodes", gen.csr_from_rows([[1], [0]])
    yield "one link", gen.csr_from_rows([[1], []])


@pytest.mark.parametrize("name,csr", list(small_cases()), ids=[n for n, _ in small_cases()])
def test_small_topologies_match_oracle_for_every_group_size(a2a, oracle, name, csr):
    rp, col = csr
    topo = a2a.Topology(rp, col)
    o = oracle.run(rp, col, threads=8)
    load, dsum, flags = all_group_sizes(a2a, topo)
    assert_loads_close(load, o.load)
    assert dsum == int(o.dist_sum.sum()) and flags == o.flags
    topo.close()


def test_source_ranges_for_every_group_size(a2a, oracle):
    """Partial source ranges (a ragged last batch, a range that starts inside a batch)."""
    rp, col = gen.random_regular(700, 4, 12)
    topo = a2a.Topology(rp, col)
    for s0, cnt in ((0, 700), (0, 1), (13, 200), (640, 60), (699, 1)):
        o = oracle.run(rp, col, s0, cnt)
        load, dsum, flags = all_group_sizes(a2a, topo, s0, cnt)
        assert_loads_close(load, o.load)
        assert dsum == int(o.dist_sum.sum()) and flags == o.flags
    topo.close()


def test_random_digraphs_for_every_group_size(a2a, oracle):
    """Seeded digraphs of no particular shape: unreachable pairs, nodes without links, parallel links."""
    for seed in range(0, 160, 4):
        rp, col = random_digraph(seed)
        if len(col) == 0:
            continue
        topo = a2a.Topology(rp, col)
        print(f"seed {seed} N={topo.N} E={topo.E}", flush=True)
        o = oracle.run(rp, col)
        load, dsum, flags = all_group_sizes(a2a, topo)
        assert_loads_close(load, o.load)
        assert dsum == int(o.dist_sum.sum()) and flags == o.flags
        topo.close()


def test_path_counts_of_a_small_group(a2a, oracle):
    """a2a_distances with path counts shares the forward kernel: one batch (eight waves per block) and all."""
    from gpu_helpers import run_distances, assert_sigma_equal
    rp, col = gen.random_regular(1500, 5, 3)
    topo = a2a.Topology(rp, col)
    o = oracle.run(rp, col, want_dist=True, want_sigma=True, threads=8)
    for max_ws in (None, topo.workspace_bytes(64, a2a.WS_SIGMA)):
        dist, sigma, dsum, unr, flags = run_distances(topo, max_ws=max_ws)
        assert np.array_equal(dist, o.dist)
        assert_sigma_equal(sigma, o.sigma)
    topo.close()
