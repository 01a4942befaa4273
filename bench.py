"""Benchmark: all-pairs BFS + EwSP link loads on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C5] [--cpu-sources S] [--graph]

One step = one pass of the whole hot path over the topology: a2a_link_loads over all N
sources (bit-parallel BFS, forward path counts, backward dependency pass, ordered reduction)
followed by a2a_schedule_bound.  The CSR is resident on the device before the timed region.
Prints one JSON line.  TEPS = N * E / seconds (one traversed edge = one (source, link) pair).

The timed region holds the K steps and nothing else.  The per-kernel split (HIP events around every
launch, on the stream the kernels run on) comes from two further, untimed steps; one more untimed
step counts the (source, link) pairs on shortest paths for the algorithmic bytes.  Beside the metric:
a plain 1 GiB device copy and fill (what this machine's HBM gives a streaming kernel), a2a_distances,
a2a_link_loads_demand, a2a_sssp_loads, and the CPU oracle on a bounded sample (all cores and one core).
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


# Profile classes of the library -> the kernel that runs them.  One k_fwd / k_bwd launch serves a level of
# every batch; the class says which lane layout the level's size stands for (every batch picks its own).
KERNEL_NAME = {"bfs": "k_bfs_level", "offsets": "k_write_offsets", "fwd_rows": "k_fwd[rows]",
               "fwd_few": "k_fwd[few]", "fwd_spread": "k_fwd[spread]", "bwd_rows": "k_bwd[rows]",
               "bwd_few": "k_bwd[few]", "bwd_spread": "k_bwd[spread]", "reduce": "k_reduce_part"}
FWD_CLASSES = ("fwd_rows", "fwd_few", "fwd_spread")
BWD_CLASSES = ("bwd_rows", "bwd_few", "bwd_spread")


def algorithmic_bytes(prof, dag_level, nb, E, steps):
    """Algorithmic bytes per kernel class for one step.

    Per reachable (source, node) pair: level tag 1 B written (BFS) + 1 B read (forward),
    sigma 8 B written (forward) + 8 B read (backward), coef 8 B written (backward) = 26 B.
    Per (source, shortest-path link): sigma gather 8 B (forward) + coef gather 8 B (backward).
    Per (batch, link): partial load 8 B written (backward, spread over its launches in
    proportion to their links) + 8 B read (ordered reduction).
    A launch at level l is charged the pairs of level l and the links into (forward) or out of
    (backward) that level; which kernel class ran the level comes from the per-level timings.
    The forward launch of the deepest level also leaves coef = 1/sigma behind (no backward
    launch there): that level's own 16 backward bytes are charged to it.
    """
    L = len(prof["pairs_level"])
    pairs = [p / steps for p in prof["pairs_level"]]       # per step
    dag_in = list(dag_level)                                # links into level l (one step)
    dag_out = [dag_in[l + 1] if l + 1 < L else 0 for l in range(L)]
    dag_total = max(sum(dag_in), 1)
    ran = {k: [ms > 0 for ms in prof[k]["ms_level"]] for k in KERNEL_NAME}
    out = {k: 0.0 for k in KERNEL_NAME}
    for l in range(L):
        if ran["bfs"][l]:
            out["bfs"] += 1 * pairs[l]
        fwd = next((k for k in ("fwd_rows", "fwd_few", "fwd_spread") if ran[k][l]), None)
        if fwd:
            out[fwd] += (1 + 8) * pairs[l] + 8 * dag_in[l]
        own = (8 + 8) * pairs[l]                      # sigma read + coef written at the node itself
        links = 8 * dag_out[l] + 8.0 * nb * E * dag_out[l] / dag_total
        bwd = next((k for k in ("bwd_rows", "bwd_few", "bwd_spread") if ran[k][l]), None)
        if bwd:
            out[bwd] += own + links
        elif fwd:  # deepest level: the forward launch leaves coef = 1/sigma, nothing runs backward
            out[fwd] += own
    out["reduce"] = 8.0 * nb * E
    return out


def layout_bytes(prof, dag_level, nb, E, steps, narrow_levels):
    """The same count with the bytes the chosen layout moves: path counts of a level kept in single precision
    (bit l+1 of narrow_levels: level l is) cost 4 bytes where the algorithmic count has 8."""
    L = len(prof["pairs_level"])
    narrow = [True] + [bool((narrow_levels >> (l + 1)) & 1) for l in range(L - 1)]
    total = 16.0 * nb * E
    for l in range(L):
        pairs = prof["pairs_level"][l] / steps
        sig = 4 if narrow[l] else 8
        total += pairs * (2 + 2 * sig + 8)
        total += dag_level[l] * ((4 if (l == 0 or narrow[l - 1]) else 8) + 8)
    return total


def read_traffic(config, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this configuration
    (profiles/<config>_pmc_traffic.txt), or None if there is none."""
    path = os.path.join(ROOT, "profiles", config.lower() + "_pmc_traffic.txt")
    if not os.path.exists(path):
        return None
    m = re.search(r"^%s\s+traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)" % re.escape(kernel),
                  open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


def copy_bandwidth(torch, reps=5):
    """Plain device-to-device copy of 1 GiB (torch's copy_ = the runtime's copy kernel): GB/s of bytes read
    plus bytes written.  What this machine's HBM gives a streaming kernel, beside the 8 TB/s data-sheet figure."""
    src = torch.ones(2 ** 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    beg, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    beg.record()
    for _ in range(reps):
        dst.copy_(src)
    end.record()
    torch.cuda.synchronize()
    ms = beg.elapsed_time(end) / reps
    beg.record()
    for _ in range(reps):
        dst.zero_()
    end.record()
    torch.cuda.synchronize()
    fill_ms = beg.elapsed_time(end) / reps
    del src, dst
    return 2.0 * 2 ** 30 / (ms * 1e-3) / 1e9, 2 ** 30 / (fill_ms * 1e-3) / 1e9


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C5")
    ap.add_argument("--cpu-sources", type=int, default=None,
                    help="sources in the oracle's timed sample (default: sized for ~10-20 s)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-distances", action="store_true",
                    help="skip the a2a_distances leg (distance matrix only, reported beside the metric)")
    ap.add_argument("--no-demand", action="store_true",
                    help="skip the a2a_link_loads_demand leg (unequal demands, reported beside the metric)")
    ap.add_argument("--no-sssp", action="store_true",
                    help="skip the a2a_sssp_loads leg (single-path SSSP baseline, reported beside the metric)")
    ap.add_argument("--sssp-iter-sources", type=int, default=512)
    ap.add_argument("--graph", action="store_true",
                    help="record a2a_link_loads into a HIP graph once and replay it in every step (the call only "
                         "enqueues kernels; small topologies are bound by launches, which a replay makes cheaper)")
    ap.add_argument("--max-workspace-gib", type=float, default=None)
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="kept for old command lines: the 1 GiB device copies (known bytes, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings) now always run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (sources would shard across GPUs with one "
              "ordered sum of E doubles at the end). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import a2a_inputs as gen
    import paper_2309_13541_amd as a2a

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    a2a.load_library()
    torch.cuda.set_device(0)
    rp, col = gen.named_config(args.config)
    t0 = time.perf_counter()
    topo = a2a.Topology(rp, col)
    t_create = time.perf_counter() - t0
    N, E = topo.N, topo.E
    cap = None if args.max_workspace_gib is None else int(args.max_workspace_gib * 2 ** 30)
    ws = topo.alloc_workspace(N, a2a.WS_LOADS, cap)
    load = torch.empty(E, dtype=torch.float64, device="cuda")
    dsum = torch.zeros(1, dtype=torch.int64, device="cuda")
    flags = torch.zeros(1, dtype=torch.int64, device="cuda")

    graph = None

    def step():
        if graph is not None:
            graph.replay()
        else:
            topo.link_loads(0, N, load=load, dist_sum_total=dsum, flags=flags, workspace=ws)
        # sum_dist / flags stay on the device until the end; the bound needs Lmax only
        return topo.schedule_bound(load, 0, 0, 1.0, 1.0)[0]

    if args.graph:
        step()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            topo.link_loads(0, N, load=load, dist_sum_total=dsum, flags=flags, workspace=ws)
        graph = g

    copy_gbps, fill_gbps = copy_bandwidth(torch)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: K steps, nothing else (no per-launch events); an event pair per step gives the median
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        bound = step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    median_ms = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    load_timed = load.clone()
    # untimed: per-kernel split from HIP events around every launch, on the stream the kernels run on
    prof_steps = 2
    graph = None  # the profiled steps are launched one by one
    topo.profile_enable(1)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = topo.profile_read()
    # one more untimed step counts the (source, link) pairs on shortest paths; its loads must be
    # the same bits as the timed step's (fixed summation order)
    topo.profile_enable(2)
    step()
    torch.cuda.synchronize()
    rerun_bitwise = bool(torch.equal(load_timed, load))
    del load_timed
    prof2 = topo.profile_read()
    dag, dag_level = prof2["dag_links"], prof2["dag_level"]
    topo.profile_enable(0)
    sec = elapsed / args.steps
    sum_dist = int(dsum.item())
    fl = int(flags.item())
    bound, _ = topo.schedule_bound(load, sum_dist, fl, 1.0, 1.0, allow_disconnected=True)

    steps = prof_steps  # the per-kernel figures come from the profiled steps
    nb = (N + 63) // 64
    alg = algorithmic_bytes(prof, dag_level, nb, E, steps)
    cfg = args.config
    per_kernel = {}
    for k, name in KERNEL_NAME.items():
        ms, n = prof[k]["ms"], prof[k]["launches"]
        if n:
            per_kernel[name] = {"ms_per_step": ms / steps, "launches_per_step": n / steps,
                                "avg_launch_ms": ms / n, "alg_GB_per_step": alg[k] / 1e9,
                                "alg_GBps": alg[k] / (ms / steps * 1e-3) / 1e9 if ms > 0 else None,
                                "ms_by_level": {str(l): round(x / steps, 3)
                                                for l, x in enumerate(prof[k]["ms_level"]) if x > 0}}
    # The dominant kernel: k_fwd and k_bwd are one kernel each (all their levels), the others as named.
    groups = {"k_bwd": BWD_CLASSES, "k_fwd": FWD_CLASSES, "k_bfs_level": ("bfs",),
              "k_write_offsets": ("offsets",), "k_reduce_part": ("reduce",)}
    g_ms = {g: sum(prof[c]["ms"] for c in cl) for g, cl in groups.items()}
    kname = max(g_ms, key=g_ms.get)
    n_l = sum(prof[c]["launches"] for c in groups[kname])
    k_alg = sum(alg[c] for c in groups[kname])            # per step
    k_ms = g_ms[kname] / steps                            # per step
    achieved = k_alg / (k_ms * 1e-3) / 1e9
    alg_total = sum(alg.values())
    lay_total = layout_bytes(prof, dag_level, nb, E, steps, prof["narrow_levels"])
    traffic = read_traffic(cfg, kname)
    # the single longest launch of that kernel (one BFS level), with its own bytes
    longest = None
    for c in groups[kname]:
        for l, x in enumerate(prof[c]["ms_level"]):
            if x > 0 and (longest is None or x > longest[2]):
                longest = (c, l, x)
    longest_launch = None
    if longest is not None and kname in ("k_fwd", "k_bwd"):
        c, l, x = longest
        one = {k: dict(v, ms_level=[m if (k == c and i == l) else 0.0 for i, m in enumerate(v["ms_level"])])
               if isinstance(v, dict) and "ms_level" in v else v for k, v in prof.items()}
        a_one = algorithmic_bytes(one, dag_level, nb, E, steps)[c]
        ms_one = x / steps
        longest_launch = {"kernel": f"{kname} level {l} ({c.split('_')[1]})", "ms": ms_one, "alg_bytes": a_one,
                          "achieved": a_one / (ms_one * 1e-3) / 1e9, "frac": a_one / (ms_one * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                          "traffic": read_traffic(cfg, f"{kname}[level {l}]")}
    roofline = {
        "bound": "hbm", "kernel": kname, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
        "alg_bytes_per_launch": k_alg * steps / n_l, "avg_launch_ms": g_ms[kname] / n_l,
        "launches_per_step": n_l / steps,
        "longest_launch": longest_launch,
        "copy_GBps": copy_gbps, "fill_GBps": fill_gbps, "frac_of_copy": achieved / copy_gbps,
        "whole_path": {"alg_bytes": alg_total, "GBps": alg_total / sec / 1e9,
                       "frac": alg_total / sec / 1e9 / HBM_PEAK_GBPS,
                       "frac_of_copy": alg_total / sec / 1e9 / copy_gbps,
                       "layout_bytes": lay_total, "layout_frac": lay_total / sec / 1e9 / HBM_PEAK_GBPS,
                       "traffic": read_traffic(cfg, "whole_step")},
        "per_kernel": per_kernel,
    }

    # the same path with a demand per pair (seeded uniform [0.5, 1.5), one double per pair), beside the metric
    dem_leg = None
    if not args.no_demand:
        gen_dev = torch.Generator(device="cuda")
        gen_dev.manual_seed(2024)
        dem = torch.rand((N, N), generator=gen_dev, dtype=torch.float64, device="cuda").add_(0.5)  # [target][source]
        dload = torch.empty(E, dtype=torch.float64, device="cuda")
        wdist = torch.zeros(1, dtype=torch.float64, device="cuda")

        def demstep():
            topo.link_loads_demand(0, N, demand=dem, load=dload, weighted_dist=wdist, workspace=ws)

        demstep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            demstep()
        torch.cuda.synchronize()
        dmsec = (time.perf_counter() - t0) / args.steps
        # every unit of demand crosses D(s,t) links: the loads must add up to demand x distance
        total, wd = float(dload.sum().item()), float(wdist.item())
        dem_leg = {"ms_per_step": dmsec * 1e3, "teps": N * E / dmsec, "unit": "edges/s",
                   "extra_alg_bytes": 8.0 * N * N, "sum_load_over_weighted_dist": total / wd if wd else None,
                   "what": "a2a_link_loads_demand over all sources, demand matrix double[N][N] resident in HBM"}
        assert wd > 0 and abs(total / wd - 1.0) < 1e-9, (total, wd)
        del dem, dload

    # single-path SSSP baseline over all sources, reported beside the metric
    sssp_leg = None
    if not args.no_sssp:
        k = max(64, args.sssp_iter_sources // 64 * 64)
        wss = torch.empty(topo.workspace_bytes(min(k, (N + 63) // 64 * 64), a2a.WS_SSSP), dtype=torch.uint8, device="cuda")
        sload = torch.empty(E, dtype=torch.float64, device="cuda")
        sdsum = torch.zeros(1, dtype=torch.int64, device="cuda")

        def sstep():
            topo.sssp_loads(0, N, k, load=sload, dist_sum_total=sdsum, workspace=wss)

        sstep()
        torch.cuda.synchronize()
        n_s = max(1, min(args.steps, 3))
        t0 = time.perf_counter()
        for _ in range(n_s):
            sstep()
        torch.cuda.synchronize()
        ssec = (time.perf_counter() - t0) / n_s
        total = float(sload.sum().item())
        assert total == float(sdsum.item()) == float(sum_dist), (total, sum_dist)  # one path of D links per pair
        sssp_leg = {"ms_per_step": ssec * 1e3, "teps": N * E / ssec, "unit": "edges/s", "iter_sources": k,
                    "max_load": float(sload.max().item()), "max_load_over_ewsp": float(sload.max().item()) / bound.max_load,
                    "what": "a2a_sssp_loads over all sources: BFS + cost recursion + path counts per iteration"}
        if not args.no_cpu:
            import oracle
            oracle.build(force=False)
            n_or = min(N, 2 * k)
            t0 = time.perf_counter()
            oracle.sssp(rp, col, 0, n_or, iter_sources=k)
            t_or = time.perf_counter() - t0
            sssp_leg["cpu_oracle"] = {"value": n_or * E / t_or, "unit": "edges/s", "cores": 1, "seconds": t_or,
                                      "sample": f"sources 0..{n_or - 1} of {N} (serial by definition)"}
        del wss, sload

    # a2a_distances alone (BFS + the int32 distance matrix), reported beside the metric
    dist_leg = None
    ws_gib = ws.numel() / 2 ** 30
    if not args.no_distances:
        del ws
        torch.cuda.empty_cache()
        wsd = topo.alloc_workspace(N, a2a.WS_DISTANCES, cap)
        dist = torch.empty((N, N), dtype=torch.int32, device="cuda")
        dsrc = torch.empty(N, dtype=torch.int64, device="cuda")
        unr = torch.zeros(1, dtype=torch.int64, device="cuda")

        def dstep():
            topo.distances(0, N, dist=dist, sigma=None, dist_sum=dsrc, unreachable=unr, flags=None, workspace=wsd)

        dstep()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            dstep()
        torch.cuda.synchronize()
        dsec = (time.perf_counter() - t0) / args.steps
        topo.profile_enable(1)
        dstep()
        dprof = topo.profile_read()
        topo.profile_enable(0)
        if fl == 0:
            assert int(dsrc.sum().item()) == sum_dist and int(unr.item()) == 0
        dist_leg = {"ms_per_step": dsec * 1e3, "teps_bfs": N * E / dsec, "unit": "edges/s",
                    "alg_bytes": 4.0 * N * N, "frac": 4.0 * N * N / dsec / 1e9 / HBM_PEAK_GBPS,
                    "kernel_ms": {k: round(dprof[k]["ms"], 3) for k in ("init", "bfs", "extract")},
                    "what": "a2a_distances over all sources: BFS + int32 dist[N][N] + per-source sums"}
        del dist, wsd

    cpu = None
    if not args.no_cpu:
        import oracle
        oracle.build(force=False)
        cores = min(os.cpu_count() or 1, 16)
        sample = args.cpu_sources
        if sample is None:
            # probe 32 sources per thread (start-up included, so it runs slow), then size the
            # sample so that the timed run takes 10-20 s
            p = min(N, 32 * cores)
            tp = time.perf_counter(); oracle.run(rp, col, 0, p, threads=cores); tp = time.perf_counter() - tp
            sample = int(max(p, min(N, p * 25.0 / max(tp, 1e-4))))
        tc = time.perf_counter()
        res = oracle.run(rp, col, 0, sample, threads=cores)
        tc = time.perf_counter() - tc
        # the same on one core, on a sample sized for about 5 s from the all-core rate
        one = int(max(1, min(N, sample * 5.0 / max(tc, 1e-4) / max(res.threads, 1))))
        t1 = time.perf_counter()
        oracle.run(rp, col, 0, one, threads=1)
        t1 = time.perf_counter() - t1
        cpu = {"value": sample * E / tc, "unit": "edges/s", "cores": res.threads, "kind": "oracle",
               "sample": f"sources 0..{sample - 1} of {N} on the same CSR ({tc:.1f} s); "
                         f"serial BFS + dependency pass per source, sources split over threads",
               "seconds": tc,
               "one_core": {"value": one * E / t1, "unit": "edges/s", "cores": 1, "seconds": t1,
                            "sample": f"sources 0..{one - 1} of {N}"}}

    out = {
        "metric": "all_pairs_bfs_link_load_teps", "value": N * E / sec, "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3,
        "ms_per_step_median": median_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": f"{args.config}: " + {
            "C1": "8x8 torus", "C2": "hypercube n=10", "C3": "16x16x16 torus",
            "C4": "Imase-Itoh N=16384 d=4", "C5": "random 8-regular digraph N=65536 seed 1234",
        }[args.config] + ", unit all-pairs demand", "N": N, "E": E, "sources": N,
            "launch": "graph replay" if args.graph else "eager", "workspace_GiB": ws_gib, "groups_per_step": prof["groups"] // max(prof["calls"], 1),
            "depth": prof["depth"], "dag_links": dag},
        "result": {"sum_dist": sum_dist, "max_load": bound.max_load, "argmax_arc": bound.argmax_arc,
                   "rerun_bitwise": rerun_bitwise, "ratio_to_lower_bound": bound.ratio, "flags": fl},
        "topo_create_ms": t_create * 1e3,
        "roofline": roofline,
        "distances": dist_leg,
        "demand": dem_leg,
        "sssp": sssp_leg,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
