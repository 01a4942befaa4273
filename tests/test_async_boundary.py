"""The compute entry points only enqueue: they return while earlier work on the stream is still running, can be
recorded into a HIP graph, and one handle serves several streams and threads at once.  Results against the
oracle / the eager call every time.  (Needs an MI355X.)"""
import threading

import numpy as np
import pytest

import a2a_inputs as gen
from gpu_helpers import run_link_loads, assert_loads_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def a2a():
    import torch
    assert torch.cuda.is_available()
    import paper_2309_13541_amd as lib
    lib.load_library()
    return lib


def test_calls_return_before_earlier_work_on_the_stream_has_finished(a2a, oracle):
    """A long spin kernel is put on the stream first; a2a_link_loads, a2a_link_loads_demand and a2a_distances are
    called behind it and must all have returned while it still runs (an event recorded right after the spin
    kernel is not yet done when the last call returns)."""
    import torch
    rp, col = gen.random_regular(1500, 5, 3)
    N = 1500
    o = oracle.run(rp, col, want_dist=True, want_sigma=True)
    topo = a2a.Topology(rp, col)
    ws = topo.alloc_workspace(N, a2a.WS_LOADS)
    ws2 = topo.alloc_workspace(N, a2a.WS_SIGMA)
    load = torch.full((topo.E,), -7.0, dtype=torch.float64, device="cuda")
    dload = torch.full((topo.E,), -7.0, dtype=torch.float64, device="cuda")
    dem = torch.ones((N, N), dtype=torch.float64, device="cuda")
    wd = torch.zeros(1, dtype=torch.float64, device="cuda")
    dsum = torch.zeros(1, dtype=torch.int64, device="cuda")
    flags = torch.zeros(1, dtype=torch.int64, device="cuda")
    dist = torch.full((N, N), -9, dtype=torch.int32, device="cuda")
    sigma = torch.full((N, N), -9.0, dtype=torch.float64, device="cuda")
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(st):
        torch.cuda._sleep(300_000_000)  # a tenth of a second of spinning at least, far longer than the calls take to enqueue
        spin_done = torch.cuda.Event()
        spin_done.record(st)
        topo.link_loads(0, N, load=load, dist_sum_total=dsum, flags=flags, workspace=ws, stream=st)
        topo.distances(0, N, dist=dist, sigma=sigma, workspace=ws2, stream=st)
        topo.link_loads_demand(0, N, demand=dem, load=dload, weighted_dist=wd, workspace=ws, stream=st)
        returned_early = not spin_done.query()
    st.synchronize()
    assert returned_early, "a compute call waited for the device"
    assert_loads_close(load.cpu().numpy(), o.load)
    assert_loads_close(dload.cpu().numpy(), o.load)
    assert int(dsum.item()) == int(o.dist_sum.sum()) and int(flags.item()) == 0
    assert float(wd.item()) == float(o.dist_sum.sum())
    assert np.array_equal(dist.cpu().numpy(), o.dist)
    assert np.array_equal(sigma.cpu().numpy(), o.sigma.astype(np.float64))
    topo.close()


def test_one_handle_two_streams_two_threads(a2a, oracle):
    """Two threads, each with its own stream, workspace and outputs, use the same handle at the same time:
    link loads of different source ranges, then a2a_schedule_bound (which reads results back) on both."""
    import torch
    rp, col = gen.random_regular(2000, 6, 8)
    topo = a2a.Topology(rp, col)
    ranges = [(0, 1100), (900, 1100)]
    want = [oracle.run(rp, col, s0, cnt) for s0, cnt in ranges]
    out = [None, None]
    errors = []
    barrier = threading.Barrier(2)

    def work(i):
        try:
            torch.cuda.set_device(0)
            s0, cnt = ranges[i]
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                ws = topo.alloc_workspace(cnt, a2a.WS_LOADS)
                load = torch.full((topo.E,), -7.0, dtype=torch.float64, device="cuda")
                dsum = torch.zeros(1, dtype=torch.int64, device="cuda")
            st.synchronize()
            barrier.wait()
            bounds = []
            for _ in range(20):
                topo.link_loads(s0, cnt, load=load, dist_sum_total=dsum, workspace=ws, stream=st)
                b, _ = topo.schedule_bound(load, 1, 0, stream=st)
                bounds.append((b.max_load, b.argmax_arc, b.min_load))
            st.synchronize()
            out[i] = (load.cpu().numpy(), int(dsum.item()), bounds)
        except Exception as e:  # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i in range(2):
        load, dsum, bounds = out[i]
        assert_loads_close(load, want[i].load)
        assert dsum == int(want[i].dist_sum.sum())
        for mx, arg, mn in bounds:  # every read-back belongs to this thread's own load vector
            assert mx == load.max() and mn == load.min() and arg == int(np.argmax(load))
    topo.close()


def test_link_loads_recorded_into_a_graph_and_replayed(a2a, oracle):
    """a2a_link_loads under stream capture: no wait, no copy, no allocation, no memset node.  The graph is
    replayed several times with other work of the program in between; every replay gives the eager bits."""
    import torch
    for rp, col in (gen.named_config("C1"), gen.random_regular(700, 4, 12)):
        topo = a2a.Topology(rp, col)
        N = topo.N
        eager, esum, eflags = run_link_loads(topo)
        assert_loads_close(eager, oracle.run(rp, col).load)
        ws = topo.alloc_workspace(N, a2a.WS_LOADS)
        load = torch.full((topo.E,), -7.0, dtype=torch.float64, device="cuda")
        dsum = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        flags = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            topo.link_loads(0, N, load=load, dist_sum_total=dsum, flags=flags, workspace=ws, stream=side)  # warm-up
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            topo.link_loads(0, N, load=load, dist_sum_total=dsum, flags=flags, workspace=ws)
        for rep in range(4):
            load.fill_(-3.0)
            ws.random_(0, 255)  # the program's own eager work between replays: scribble over everything
            dsum.fill_(-5)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(load.cpu().numpy(), eager), rep
            assert int(dsum.item()) == esum and int(flags.item()) == eflags
        del graph
        topo.close()


def test_large_disconnected_topology_needs_no_oversized_workspace(a2a, oracle):
    """Two 4096-node components: some pairs have no path, the deepest BFS level is still small, and the level
    slots of the workspace follow it (they used to be sized for N levels)."""
    a_rp, a_col = gen.random_regular(4096, 4, 31)
    b_rp, b_col = gen.hypercube(12)
    rows = [list(a_col[a_rp[u]:a_rp[u + 1]]) for u in range(4096)]
    rows += [[4096 + int(w) for w in b_col[b_rp[u]:b_rp[u + 1]]] for u in range(4096)]
    rp, col = gen.csr_from_rows(rows)
    topo = a2a.Topology(rp, col)
    assert topo.level_bound == 12  # the hypercube half; the random half is shallower
    assert topo.workspace_bytes(topo.N, a2a.WS_LOADS) < 2 * 2 ** 30
    o = oracle.run(rp, col, threads=16)
    load, dsum, flags = run_link_loads(topo)
    assert flags == a2a.FLAG_UNREACHABLE == o.flags and dsum == int(o.dist_sum.sum())
    assert_loads_close(load, o.load)
    import torch
    b, st = topo.schedule_bound(torch.from_numpy(load).cuda(), dsum, flags, allow_disconnected=True)
    assert st == a2a.ERR_DISCONNECTED
    topo.close()
