"""a2a_link_loads_static (the entry point that allocates nothing on the device) against a2a_link_loads through
the C ABI: two calls in a row on the library's fixed workspace array, the second with a smaller input, then a
topology that does not fit."""
import ctypes

import numpy as np
import pytest

import a2a_inputs as gen

pytestmark = pytest.mark.gpu


def _raw_static(lib, topo, s0, cnt, load, dsum, flags, stream=None):
    return lib.a2a_link_loads_static(topo._h, s0, cnt, load.data_ptr(), dsum.data_ptr(), flags.data_ptr(), stream)


def test_static_workspace_matches_link_loads_twice_in_a_row(oracle):
    import torch
    import paper_2309_13541_amd as a2a
    from gpu_helpers import run_link_loads, assert_loads_close
    lib = a2a.load_library()
    big = gen.random_regular(3000, 6, 77)      # 47 batches: several groups inside the 32 MiB array
    small = gen.torus([5, 13])                 # N = 65: two batches, one group
    results = []
    for rp, col, s0, cnt in ((*big, 0, 3000), (*small, 3, 60)):
        topo = a2a.Topology(rp, col)
        print(f"case N={topo.N} E={topo.E} sources {s0}+{cnt}", flush=True)
        assert topo.workspace_bytes(cnt, a2a.WS_LOADS | a2a.WS_MINIMAL) <= a2a.STATIC_WORKSPACE_BYTES
        load = torch.full((topo.E,), -7.0, dtype=torch.float64, device="cuda")
        dsum = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        flags = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        # no allocation through torch (its count of allocations stands still; the bytes in use may drop at any
        # time, when Python collects what earlier tests left behind) and none on the device beside it
        torch.cuda.synchronize()
        allocs = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
        free_before = torch.cuda.mem_get_info()[0]
        st = _raw_static(lib, topo, s0, cnt, load, dsum, flags)
        torch.cuda.synchronize()
        assert st == a2a.OK
        assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == allocs
        assert torch.cuda.mem_get_info()[0] >= free_before
        got = load.cpu().numpy()
        # the existing entry point with a caller-owned workspace of the same size: same groups, same order
        ws = torch.empty(a2a.STATIC_WORKSPACE_BYTES, dtype=torch.uint8, device="cuda")
        want, wsum, wflags = run_link_loads(topo, s0, cnt, workspace=ws)
        assert np.array_equal(got, want)
        assert int(dsum.item()) == wsum and int(flags.item()) == wflags
        # and both against the oracle, to the bar of the parity tests
        o = oracle.run(rp, col, s0, cnt)
        assert_loads_close(got, o.load)
        assert wsum == int(o.dist_sum.sum())
        results.append(got)
        topo.close()
    assert len(results) == 2


def test_static_workspace_refuses_what_does_not_fit():
    import torch
    import paper_2309_13541_amd as a2a
    lib = a2a.load_library()
    rp, col = gen.ring(40000)  # 40 000 BFS levels x 40 000 nodes: far beyond 32 MiB for one batch
    topo = a2a.Topology(rp, col)
    assert topo.workspace_bytes(64, a2a.WS_LOADS | a2a.WS_MINIMAL) > a2a.STATIC_WORKSPACE_BYTES
    load = torch.full((topo.E,), -7.0, dtype=torch.float64, device="cuda")
    dsum = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    flags = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    assert _raw_static(lib, topo, 0, 64, load, dsum, flags) == a2a.ERR_WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
    assert float(load.min().item()) == -7.0  # nothing was enqueued
    with pytest.raises(a2a.A2AError) as e:
        topo.link_loads_static(0, 64, load=load)
    assert e.value.status == a2a.ERR_WORKSPACE_TOO_SMALL
    assert lib.a2a_link_loads_static(None, 0, 1, load.data_ptr(), None, None, None) == a2a.ERR_INVALID_ARG
    topo.close()
