"""Helpers for the GPU parity tests: run the C-ABI entry points and bring results to numpy."""
import numpy as np


def run_link_loads(topo, src_begin=0, src_count=None, max_ws=None, workspace=None):
    import torch
    import paper_2309_13541_amd as a2a
    if src_count is None:
        src_count = topo.N - src_begin
    ws = workspace if workspace is not None else topo.alloc_workspace(src_count, a2a.WS_LOADS, max_ws)
    load = torch.full((max(topo.E, 1),), -7.0, dtype=torch.float64, device="cuda")
    dsum = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    flags = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    topo.link_loads(src_begin, src_count, load=load, dist_sum_total=dsum, flags=flags, workspace=ws)
    torch.cuda.synchronize()
    return load[:topo.E].cpu().numpy(), int(dsum.item()), int(flags.item())


def run_distances(topo, src_begin=0, src_count=None, want_sigma=True, want_dist=True, max_ws=None):
    import torch
    import paper_2309_13541_amd as a2a
    if src_count is None:
        src_count = topo.N - src_begin
    fl = a2a.WS_SIGMA if want_sigma else a2a.WS_DISTANCES
    ws = topo.alloc_workspace(src_count, fl, max_ws)
    rows = max(src_count, 1)
    dist = torch.full((rows, topo.N), -9, dtype=torch.int32, device="cuda") if want_dist else None
    sigma = torch.full((rows, topo.N), -9.0, dtype=torch.float64, device="cuda") if want_sigma else None
    dsum = torch.full((rows,), -1, dtype=torch.int64, device="cuda")
    unr = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    flags = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    topo.distances(src_begin, src_count, dist=dist, sigma=sigma, dist_sum=dsum, unreachable=unr,
                   flags=flags, workspace=ws)
    torch.cuda.synchronize()
    return (dist[:src_count].cpu().numpy() if want_dist else None,
            sigma[:src_count].cpu().numpy() if want_sigma else None,
            dsum[:src_count].cpu().numpy(), int(unr.item()), int(flags.item()))


def assert_loads_close(got, want, rtol=1e-9):
    """|gpu - oracle| <= rtol * |oracle| for every link (fp64 loads, bar: relative 1e-9)."""
    got = np.asarray(got); want = np.asarray(want)
    assert got.shape == want.shape
    err = np.abs(got - want)
    bad = err > rtol * np.abs(want)
    assert not bad.any(), (f"{bad.sum()} of {bad.size} links off; worst rel "
                           f"{(err / np.maximum(np.abs(want), 1e-300)).max():.3e} at {int(np.argmax(err))}")


def assert_sigma_equal(got_f64, want_u64):
    """Path counts below 2^53 must match bit for bit."""
    want = np.asarray(want_u64)
    assert want.max(initial=0) < 2 ** 53
    assert np.array_equal(np.asarray(got_f64), want.astype(np.float64))
