/*
 * a2a_topo -- all-to-all evaluation of a direct-connect topology on one AMD MI355X.
 *
 * The topology is the directed graph G=(V,E) of Sec. 2.2 of the paper (|V| = N hosts,
 * out-degree d, link bandwidth b), handed over as an int32 out-neighbour CSR.  Every CSR
 * entry is one link; its position is the link id.  The library computes, entirely in HIP
 * kernels on the device:
 *   - hop distances D(s,t) (the D(.,.) of Theorem 1, Sec. 5.4) and the number sigma(s,t)
 *     of distinct shortest link sequences ("all the shortest paths", Sec. 5.2);
 *   - the Equal-weight Shortest Path (EwSP) link loads of Sec. 5.2 / 5.3: every ordered
 *     pair carries unit demand, split equally over all of its shortest paths;
 *   - the schedule figures that follow: all-to-all time = maximum link load (Sec. 5.3)
 *     scaled by m/b, the capacity lower bound of Eq. (lb) (Theorem 1), throughput
 *     (N-1)m/T (Sec. 2.2) and its upper bound (N-1) f b (Sec. 5.1).
 *
 * Conventions
 *   - "host" / "device" after a pointer says where the memory lives.  The caller owns every
 *     buffer and the stream; the library owns only the opaque handle (a device copy of the
 *     out- and in-neighbour CSR, a few KB of pinned host memory).
 *   - All device work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  a2a_distances, a2a_link_loads, a2a_link_loads_demand and
 *     a2a_link_loads_static only enqueue kernels of this library: they never wait for the device,
 *     copy nothing to the host and allocate nothing, so they return while earlier work on the
 *     stream may still be running, and a stream under HIP graph capture records them (the launch
 *     sequence depends only on the handle, the source range and the workspace size; what depends
 *     on the data is decided inside the kernels).  Exception: while a2a_profile_enable is on they
 *     wait, to read counters back.  a2a_schedule_bound / _cap wait for their result; a2a_topo_create
 *     runs a breadth-first search from every node on the default stream and waits for it.
 *   - A handle may be used from several threads and streams at once, each call with its own
 *     workspace and outputs (up to 64 a2a_schedule_bound / _cap calls in flight per handle);
 *     a2a_profile_enable / _read are not thread safe.
 *   - Every function returns an a2a_status (0 = A2A_OK, negative = error); nothing throws,
 *     aborts or prints.  On error the outputs are unspecified.
 *   - Sources are processed in batches of 64 (one bit of a 64-bit mask per source); several
 *     batches advance level by level together, as many as the workspace holds.
 *   - All arithmetic is in double precision.  Inside the workspace the path counts of BFS level
 *     l are kept as floats while (largest in-degree)^l < 2^24, i.e. while every one of them is
 *     certain to be a whole number that a float holds exactly; results do not depend on it.
 */
#ifndef A2A_TOPO_H
#define A2A_TOPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct a2a_topo a2a_topo;

typedef enum a2a_status {
  A2A_OK = 0,
  A2A_ERR_INVALID_ARG = -1,         /* null pointer, N <= 0, malformed CSR, bad source range */
  A2A_ERR_SELF_LOOP = -2,           /* a link u -> u (generators drop them before create) */
  A2A_ERR_WORKSPACE_TOO_SMALL = -3, /* workspace cannot hold one batch of 64 sources */
  A2A_ERR_HIP = -4,                 /* a HIP runtime call failed (no device, out of memory ...) */
  A2A_ERR_NOT_IMPLEMENTED = -5,     /* N above 4 194 304 nodes (32-bit offsets into a batch's arrays) */
  A2A_ERR_DISCONNECTED = -6,        /* some ordered pair has no path: all-to-all infeasible */
  A2A_ERR_NO_MEMORY = -7,           /* host allocation failed */
  A2A_ERR_LEVEL_OVERFLOW = -8       /* not returned any more (the handle knows the deepest BFS level) */
} a2a_status;

/* flags of a2a_workspace_bytes */
#define A2A_WS_DISTANCES 0x0 /* a2a_distances without sigma */
#define A2A_WS_SIGMA 0x1     /* a2a_distances with sigma */
#define A2A_WS_LOADS 0x2     /* a2a_link_loads */
#define A2A_WS_SSSP 0x4      /* a2a_sssp_loads; pass iter_sources as src_count */
#define A2A_WS_MINIMAL 0x100 /* smallest usable size (one batch at a time) instead of the
                                recommended one (all batches advance together) */

/* bits written to *flags by a2a_distances / a2a_link_loads */
#define A2A_FLAG_SIGMA_INEXACT 0x1 /* some path count reached 2^53: sigma no longer exact */
#define A2A_FLAG_UNREACHABLE 0x2   /* some ordered pair (s,t), t != s, has no path */

/*
 * Validates the CSR, builds the in-neighbour CSR (stable in link-id order) and uploads both.
 *   N        number of hosts, 0 < N <= 4 194 304 (more: A2A_ERR_NOT_IMPLEMENTED)
 *   row_ptr  host, int32[N+1], row_ptr[0] = 0, non-decreasing, row_ptr[N] = E (E may be 0)
 *   col_idx  host, int32[E], each in [0,N); parallel links allowed, self-loops rejected
 *   out      receives the handle; release with a2a_topo_destroy
 * Validation happens before the first HIP call, so malformed input is reported as
 * A2A_ERR_INVALID_ARG / A2A_ERR_SELF_LOOP even on a machine without a GPU.
 * The handle also records the largest finite D(s,t) over all ordered pairs ("level bound"; the
 * diameter if G is strongly connected), found by a breadth-first search from every node on the
 * device (about 1 GiB of temporary device memory at most, freed before returning).  It fixes the
 * number of BFS levels, hence kernel launches and workspace level slots, of every later call.
 */
int a2a_topo_create(int32_t N, const int32_t* row_ptr, const int32_t* col_idx, a2a_topo** out);

/* Frees the handle and its device memory.  NULL is ignored. */
void a2a_topo_destroy(a2a_topo* topo);

/* Any output pointer may be NULL.  dmax = largest out-degree. */
int a2a_topo_info(const a2a_topo* topo, int32_t* N, int64_t* E, int32_t* dmax, int32_t* level_bound);

/*
 * Bytes of device workspace for a call over src_count sources.  With A2A_WS_MINIMAL the
 * smallest size the call accepts; otherwise the size at which all ceil(src_count/64) batches
 * advance together (fewest kernel launches).  Any size in between is used as well as it can
 * be.  Returns 0 on bad arguments.  The workspace must be 256-byte aligned.
 */
size_t a2a_workspace_bytes(const a2a_topo* topo, int32_t src_count, int flags);

/*
 * Hop distances (and optionally shortest-path counts) from sources
 * src_begin .. src_begin+src_count-1 to every node: D(s,t) of Theorem 1 (Sec. 5.4) by
 * bit-parallel breadth-first search, sigma(s,t) by level-ordered accumulation over the
 * links that lie on shortest paths (Sec. 5.2).
 *   dist         device, int32[src_count][N], row-major; -1 = unreachable.  May be NULL.
 *   sigma        device, double[src_count][N]; exact integers below 2^53, 0 = unreachable.
 *                May be NULL (then no path counting is done).
 *   dist_sum     device, int64[src_count]: sum_t D(s,t) over reachable t.  May be NULL.
 *   unreachable  device, int64[1]: number of pairs (s,t), t != s, without a path. May be NULL.
 *   flags        device, int64[1]: A2A_FLAG_* bits.  May be NULL.
 *   workspace    device, workspace_bytes bytes (see a2a_workspace_bytes), 256-byte aligned
 */
int a2a_distances(const a2a_topo* topo, int32_t src_begin, int32_t src_count, int32_t* dist,
                  double* sigma, int64_t* dist_sum, int64_t* unreachable, int64_t* flags,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * EwSP link loads (Sec. 5.2, Sec. 5.3) of the unit demands whose source lies in
 * src_begin .. src_begin+src_count-1 (0, N = the full all-to-all):
 *   load[a] = sum_s sum_{t != s} (# shortest s->t paths through link a) / sigma(s,t).
 * Computed per source batch by a forward path-count pass and a backward dependency pass over
 * the shortest-path DAG; batch results are added in ascending batch order and every sum is taken
 * in a fixed order, so the result is bitwise reproducible from run to run and does not depend on
 * the workspace size (the size decides which batches advance together, never the order of a sum:
 * every batch picks its kernels' lane layout from its own level sizes).
 *   load            device, double[E], overwritten
 *   dist_sum_total  device, int64[1]: sum over these sources of sum_t D(s,t).  May be NULL.
 *   flags           device, int64[1]: A2A_FLAG_* bits.  May be NULL.
 */
int a2a_link_loads(const a2a_topo* topo, int32_t src_begin, int32_t src_count, double* load,
                   int64_t* dist_sum_total, int64_t* flags, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/*
 * a2a_link_loads for callers that cannot allocate device memory or bring a workspace: code under
 * HIP graph capture set-up, tight serving loops, harnesses that forbid hipMalloc.  The workspace is
 * a fixed array of A2A_STATIC_WORKSPACE_BYTES inside the library (one per GPU, held until the
 * process ends; its address is looked up once, in a2a_topo_create); the call itself allocates
 * nothing on the device and frees nothing.  Same arguments, results and reproducibility as
 * a2a_link_loads (the batches advance in as many groups as the array holds).  A2A_ERR_WORKSPACE_TOO_SMALL, before anything is enqueued, if the array cannot hold
 * one batch of this topology (a2a_workspace_bytes(topo, src_count, A2A_WS_LOADS | A2A_WS_MINIMAL)
 * tells: about 0.9 KB per node and BFS level).  All calls on one GPU share the array, whatever
 * the handle or stream: it keeps the previous call's contents (everything read is written first),
 * and two such calls that overlap in time on one GPU race; serialise them.
 */
#define A2A_STATIC_WORKSPACE_BYTES (32u << 20)
int a2a_link_loads_static(const a2a_topo* topo, int32_t src_begin, int32_t src_count, double* load,
                          int64_t* dist_sum_total, int64_t* flags, void* hip_stream);

/*
 * The same for commodities of unequal demand.  The paper's commodities all have the same
 * demand (Sec. 3.1.1); here the pair (s,t) carries demand(s,t), split equally over its
 * shortest paths as before (Sec. 5.2):
 *   load[a] = sum_s sum_{t != s} demand(s,t) * (# shortest s->t paths through link a) / sigma(s,t),
 * i.e. demand(s,t) takes the place of the unit that target t contributes in the dependency
 * recursion of a2a_link_loads.  Divide by link capacities with a2a_schedule_bound_cap.
 *   demand          device, double[N][src_count], by target: demand[t * src_count + (s - src_begin)]
 *                   is what source s sends to node t (the 64 sources of a batch lie next to each
 *                   other).  Expected finite and >= 0, not checked; demand(s,s) and the demand of
 *                   pairs without a path are ignored.  Read only.
 *   load            device, double[E], overwritten
 *   weighted_dist   device, double[1]: sum over reachable pairs of demand(s,t) * D(s,t), the
 *                   link-time the demands need at least (what sum D is for unit demands in the
 *                   capacity argument of Theorem 1).  May be NULL.
 *   dist_sum_total, flags, workspace, stream: as for a2a_link_loads (same workspace size).
 * Reproducible like a2a_link_loads.  A2A_ERR_INVALID_ARG for demand == NULL.
 */
int a2a_link_loads_demand(const a2a_topo* topo, int32_t src_begin, int32_t src_count,
                          const double* demand, double* load, double* weighted_dist,
                          int64_t* dist_sum_total, int64_t* flags, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/*
 * Link loads of the single-path baseline "SSSP" of Sec. 5.2: a heuristic that computes shortest
 * paths iteration by iteration through a graph whose link weights reflect the congestion caused
 * by the earlier iterations; every commodity (s,t) is routed over ONE path.  The paper names the
 * heuristic and cites its source but gives neither the weights nor what an iteration is; this
 * library's reading:
 *   - an iteration routes the commodities of iter_sources consecutive sources against the weights
 *     it starts with; the weight of a link is the number of commodities that the earlier
 *     iterations routed over it (0 everywhere in the first);
 *   - the path of (s,t) has D(s,t) links (hop count first, as for EwSP), among those the least
 *     total weight, among those the lowest id of the last link, then of the one before it, ...;
 *     the paths from one source form a tree;
 *   - load[a] = number of commodities with source in src_begin .. src_begin+src_count-1 routed over a.
 *   iter_sources  a positive multiple of 64 (one or more batches of 64 sources; the iterations of
 *                 a call are its groups of batches, in ascending source order).  Larger values
 *                 mean fewer, cheaper iterations and weights that react later.
 *   load          device, double[E], overwritten: whole numbers, exact
 *   dist_sum_total, flags   as for a2a_link_loads (A2A_FLAG_SIGMA_INEXACT is never set)
 *   workspace     device, at least a2a_workspace_bytes(topo, iter_sources, A2A_WS_SSSP) bytes: it must
 *                 hold a whole iteration (else A2A_ERR_WORKSPACE_TOO_SMALL); more is not used
 * Only enqueues, like a2a_link_loads.  All sums are integer: results do not depend on any order.
 * Feed load to a2a_schedule_bound for the all-to-all time of the routing (its largest link load,
 * Sec. 5.3).  A2A_ERR_INVALID_ARG if iter_sources is not a positive multiple of 64.
 */
int a2a_sssp_loads(const a2a_topo* topo, int32_t src_begin, int32_t src_count, int32_t iter_sources,
                   double* load, int64_t* dist_sum_total, int64_t* flags, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

typedef struct a2a_bound {
  double max_load;         /* Lmax: all-to-all time under unit demand and capacity (Sec. 5.3) */
  int64_t argmax_arc;      /* lowest link id whose load equals max_load */
  double min_load;
  int64_t sum_dist;        /* as passed in */
  int64_t n_links;         /* E */
  int32_t n_nodes;         /* N */
  int32_t dmax;            /* largest out-degree */
  double t_sched;          /* Lmax * m / b */
  double t_lb_nd;          /* sum_dist * m / (N * dmax * b): Eq. (lb) summed over all sources */
  double t_lb_links;       /* sum_dist * m / (E * b): same argument with the true link count */
  double ratio;            /* t_sched / t_lb_nd */
  double throughput;       /* (N-1) * m / t_sched (Sec. 2.2) */
  double flow_value;       /* f = 1 / Lmax (Sec. 5.3) */
  double throughput_upper; /* (N-1) * f * b (Sec. 5.1) */
} a2a_bound;

/*
 * Schedule completion time and bounds from the link loads.
 *   load       device, double[E] as written by a2a_link_loads over all N sources
 *   sum_dist   sum over all ordered pairs of D(s,t) (dist_sum_total of that call)
 *   flags      the A2A_FLAG_* bits of that call; if A2A_FLAG_UNREACHABLE is set the
 *              function fills `out` and returns A2A_ERR_DISCONNECTED
 *   m_bytes    shard size m (Sec. 2.2); b_bytes_per_s link bandwidth b.  m = b = 1 gives the
 *              unit-demand, unit-capacity quantities of Sec. 5.3.
 *   out        host
 * The max / argmax / min reduction runs on the device; the function waits for it.
 */
int a2a_schedule_bound(const a2a_topo* topo, const double* load, int64_t sum_dist, int64_t flags,
                       double m_bytes, double b_bytes_per_s, a2a_bound* out, void* hip_stream);

/*
 * The same for a network G = (V, E, cap) with link capacities, the general form of the problem
 * (Sec. 3.1.1, and the remark on non-uniform link bandwidth in the time-stepped LP there):
 * the flows of a routing fit when every link's load times the common rate stays within its
 * capacity, so the all-to-all time of the EwSP routing is the largest utilisation load[a] / cap[a].
 * cap[a] is the bandwidth of link a in units of b (cap = 1 everywhere gives a2a_schedule_bound).
 *   cap        device, double[E], every entry positive and finite (else A2A_ERR_INVALID_ARG,
 *              found on the device, `out` untouched)
 *   other arguments as a2a_schedule_bound
 * The capacity bound of Eq. (lb) is reported against the true total capacity (t_lb_links) and, as
 * "d x N", against N nodes of the largest total out-capacity (t_lb_nd).  The total capacity is
 * summed in a fixed order (reproducible from run to run).
 */
typedef struct a2a_bound_cap {
  double max_util;          /* Umax = max_a load[a] / cap[a] */
  int64_t argmax_arc;       /* lowest link id whose utilisation equals max_util */
  double min_util;
  int64_t sum_dist;         /* as passed in */
  int64_t n_links;          /* E */
  int32_t n_nodes;          /* N */
  int32_t reserved;
  double total_capacity;    /* sum_a cap[a] */
  double max_node_capacity; /* largest sum of cap over the out-links of one node */
  double t_sched;           /* Umax * m / b */
  double t_lb_nd;           /* sum_dist * m / (N * max_node_capacity * b) */
  double t_lb_links;        /* sum_dist * m / (total_capacity * b) */
  double ratio;             /* t_sched / t_lb_nd */
  double throughput;        /* (N-1) * m / t_sched (Sec. 2.2) */
  double flow_value;        /* f = 1 / Umax */
  double throughput_upper;  /* (N-1) * f * b (Sec. 5.1) */
} a2a_bound_cap;
int a2a_schedule_bound_cap(const a2a_topo* topo, const double* load, const double* cap, int64_t sum_dist,
                           int64_t flags, double m_bytes, double b_bytes_per_s, a2a_bound_cap* out,
                           void* hip_stream);

/*
 * Lower bound of Theorem 1 (Sec. 5.4) for any topology with N hosts and out-degree d: a source
 * reaches at most d^l hosts in l hops, so sum_t D(r,t) >= S_min(N,d), the distance sum of the
 * arborescence that fills level l with d^l hosts until all N are placed, and by Eq. (lb) the
 * all-to-all takes at least S_min * m / (d * b).  For N = (d^k - 1)/(d - 1) (full k-layer tree)
 * S_min = (d^(k+1) (k-1) - d^k k + d) / (d-1)^2.  Host arithmetic only; no device is touched.
 * Dividing the measured sum of distances (a2a_distances / a2a_link_loads) by N * s_min tells how
 * close a topology comes to the bound (generalized Kautz graphs approach 1, Sec. 5.4).
 * Returns A2A_ERR_INVALID_ARG for N < 1, d < 1 (d = 1 with N > 2^31 hosts cannot occur), m <= 0, b <= 0.
 */
typedef struct a2a_tree_bound {
  int64_t s_min;        /* distance sum of the fullest d-ary arborescence on N hosts */
  int32_t height;       /* its deepest level */
  int32_t full;         /* 1 if every level is full (closed form of Theorem 1 applies) */
  double t_lb;          /* s_min * m / (d * b) */
  double throughput_ub; /* (N-1) * m / t_lb (Sec. 2.2); 0 for N = 1 */
} a2a_tree_bound;
int a2a_tree_lower_bound(int32_t N, int32_t d, double m_bytes, double b_bytes_per_s, a2a_tree_bound* out);

/*
 * Optional per-kernel timing, for benchmarks (not part of the paper's method).
 * a2a_profile_enable(topo, mode) clears what was gathered so far and sets the mode:
 *   0  off (default);
 *   1  every kernel launch of a2a_distances / a2a_link_loads on this handle is bracketed by two
 *      HIP events on the caller's stream (a few microseconds per launch);
 *   2  as 1, and the forward pass also counts the (source, link) pairs that lie on shortest
 *      paths (one atomic per wavefront: slows the forward kernels down, use on untimed runs).
 * a2a_profile_read waits for the device and sums the event times per kernel class; index
 * A2A_K_* into ms[] / launches[].  One launch serves a level of all batches of a group and every
 * batch picks its own lane layout inside it; a launch is filed under the layout that the group's
 * average level size stands for (FWD_ROWS / FWD_FEW / FWD_SPREAD, BWD_...).  While a mode other
 * than 0 is on, the compute calls wait for the device to read counters back.  Not thread safe.
 */
typedef enum a2a_prof_kernel {
  A2A_K_INIT = 0,  /* level 0 set-up */
  A2A_K_BFS,       /* one BFS level */
  A2A_K_OFFSETS,   /* row offsets of the level-compact arrays */
  A2A_K_FWD_ROWS,  /* forward level, one wave per node (well-filled level) */
  A2A_K_FWD_FEW,   /* forward level with few sources per node: lanes = (node, link) or (node, source) */
  A2A_K_FWD_SPREAD, /* forward level, many sources per node, short rows on the level before */
  A2A_K_BWD_ROWS,  /* backward level, one wave per node */
  A2A_K_BWD_FEW,   /* backward level, lanes = (node, link) or (node, source) */
  A2A_K_BWD_SPREAD, /* backward level, many sources per node, short rows on the level after */
  A2A_K_REDUCE,    /* ordered sum of the per-batch link loads */
  A2A_K_EXTRACT,   /* dist / sigma output of a2a_distances */
  A2A_K_COUNT
} a2a_prof_kernel;
#define A2A_PROF_MAX_LEVELS 64 /* deeper levels are lumped into the last slot */
typedef struct a2a_profile {
  double ms[16];                               /* summed kernel time per a2a_prof_kernel, milliseconds */
  int64_t launches[16];                        /* launches per a2a_prof_kernel */
  double ms_level[16][A2A_PROF_MAX_LEVELS];    /* the same time split by BFS level */
  int64_t pairs_level[A2A_PROF_MAX_LEVELS];    /* reachable (source, node) pairs per level, all calls */
  int64_t dag_level[A2A_PROF_MAX_LEVELS];      /* mode 2: (source, link) pairs with D(s,w) = D(s,u)+1 = level */
  int64_t dag_links;                           /* mode 2: sum of dag_level */
  int64_t calls;                               /* a2a_distances + a2a_link_loads calls since enable */
  int32_t depth;                               /* deepest BFS level seen */
  int32_t groups;                              /* batch groups processed */
  uint64_t narrow_levels;                      /* bit l: a forward launch of level l (< 64) read the path
                                                  counts of level l-1 in single precision (the library
                                                  keeps them so while (largest in-degree)^level < 2^24:
                                                  exact, half the bytes) */
  uint64_t fwd_flavours;                       /* lane layouts the batches' forward levels picked: bit
                                                  3 * layout + p, layout 0 rows, 1 spread, 2 (node, source),
                                                  3 (node, link); p = 0 float -> float, 1 float -> double,
                                                  2 double -> double path counts */
  uint64_t bwd_flavours;                       /* the same backward: bit 2 * layout + p, p = 0 float,
                                                  1 double path counts on the level */
} a2a_profile;
int a2a_profile_enable(a2a_topo* topo, int mode);
int a2a_profile_read(a2a_topo* topo, a2a_profile* out);

/* Static string for a status code. */
const char* a2a_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* A2A_TOPO_H */
