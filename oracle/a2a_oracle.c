/*
 * CPU oracle for the all-to-all topology evaluator.  TEST INFRASTRUCTURE ONLY:
 * it may be called from tests/, from the smoke check and from the benchmark's
 * cpu_baseline leg; the product library never links, loads or calls it, and it
 * shares no code, header or table with the HIP path.
 *
 * What it computes (plain definitions, serial per source, fp64 / exact integers):
 *   D(s,t)      hop distance on the directed topology G=(V,E) of Sec. 2.2, the
 *               quantity D(.,.) used in the proof of Theorem 1 (Sec. 5.4);
 *   sigma(s,t)  number of distinct shortest s->t link sequences ("all the
 *               shortest paths" of the EwSP baseline, Sec. 5.2); every CSR entry
 *               is its own link, so parallel arcs give distinct paths;
 *   load[a]     EwSP link load: every ordered pair (s,t) carries unit demand split
 *               equally over all its shortest paths (Sec. 5.2, Sec. 5.3), so
 *               load[a] = sum_{s,t} (#shortest s->t paths through a) / sigma(s,t);
 *   bound       all-to-all time = maximum link load under unit demand and capacity
 *               (Sec. 5.3), the capacity lower bound sum D / (N d) from Eq. (lb)
 *               of Theorem 1 summed over all sources, and the throughput formulas
 *               (N-1) m / T (Sec. 2.2) and (N-1) f b (Sec. 5.1).
 *
 * Method: queue BFS from each source over the out-neighbour CSR, path counts
 * accumulated in BFS order, then the dependency recursion walked in reverse BFS
 * order (a node's successors on shortest paths are one level deeper, hence final
 * when it is visited).  Threads only split the source range; each owns a private
 * load vector and the vectors are merged in thread order.
 *
 * Pins (tests/test_oracle_*.py, tests/test_capacities.py, tests/test_demands.py): torus / hypercube /
 * K4,4 closed forms, the 3x3x3-torus flow value 1/9 of Sec. 5.1, flow-conservation and level-cut
 * invariants, exact brute-force path enumeration for N <= 12 (with unit and with unequal demands).
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define A2A_ORACLE_SIGMA_LIMIT (1ULL << 53)

/* Scratch for one source. */
typedef struct {
  int32_t* dist;   /* [N]  -1 = unreachable */
  uint64_t* sigma; /* [N] */
  double* delta;   /* [N] */
  int32_t* order;  /* [N] BFS visiting order, doubles as the FIFO queue */
} src_scratch;

/*
 * One source.  Fills sc->dist / sc->sigma, adds this source's contribution to
 * load[] (if non-NULL).  Returns sum_t D(s,t) over reachable t; *reached gets the
 * number of reachable nodes other than s; *overflow is set when a path count
 * reaches 2^53 (no longer exact in fp64).
 */
static int64_t one_source(int32_t N, const int32_t* row_ptr, const int32_t* col, int32_t s,
                          src_scratch* sc, double* load, int64_t* reached, int* overflow) {
  int32_t head = 0, tail = 0;
  int64_t dsum = 0;
  for (int32_t v = 0; v < N; ++v) {
    sc->dist[v] = -1;
    sc->sigma[v] = 0;
    sc->delta[v] = 0.0;
  }
  sc->dist[s] = 0;
  sc->sigma[s] = 1;
  sc->order[tail++] = s;
  while (head < tail) {
    int32_t u = sc->order[head++];
    for (int32_t a = row_ptr[u]; a < row_ptr[u + 1]; ++a) {
      int32_t w = col[a];
      if (sc->dist[w] < 0) {
        sc->dist[w] = sc->dist[u] + 1;
        dsum += sc->dist[w];
        sc->order[tail++] = w;
      }
      if (sc->dist[w] == sc->dist[u] + 1) {
        sc->sigma[w] += sc->sigma[u];
        if (sc->sigma[w] >= A2A_ORACLE_SIGMA_LIMIT) *overflow = 1;
      }
    }
  }
  *reached = (int64_t)tail - 1;
  if (load) {
    for (int32_t i = tail - 1; i >= 0; --i) {
      int32_t u = sc->order[i];
      for (int32_t a = row_ptr[u]; a < row_ptr[u + 1]; ++a) {
        int32_t w = col[a];
        if (sc->dist[w] == sc->dist[u] + 1) {
          /* share of the traffic arriving at (and destined to) w that came over link a */
          double c = (double)sc->sigma[u] / (double)sc->sigma[w] * (1.0 + sc->delta[w]);
          load[a] += c;
          sc->delta[u] += c;
        }
      }
    }
  }
  return dsum;
}

typedef struct {
  int32_t N;
  const int32_t* row_ptr;
  const int32_t* col;
  int32_t s_begin, s_end; /* this thread's sources */
  int32_t s_base;         /* first source of the whole call (row 0 of the outputs) */
  int32_t* dist_out;
  uint64_t* sigma_out;
  double* load;           /* private [E] or NULL */
  int64_t* dist_sum;
  int64_t unreachable;
  int overflow;
  int failed;
} job;

static void* worker(void* p) {
  job* j = (job*)p;
  int32_t N = j->N;
  src_scratch sc;
  sc.dist = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  sc.sigma = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)N);
  sc.delta = (double*)malloc(sizeof(double) * (size_t)N);
  sc.order = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  if (!sc.dist || !sc.sigma || !sc.delta || !sc.order) {
    j->failed = 1;
  } else {
    for (int32_t s = j->s_begin; s < j->s_end; ++s) {
      int64_t reached = 0;
      int64_t ds = one_source(N, j->row_ptr, j->col, s, &sc, j->load, &reached, &j->overflow);
      size_t row = (size_t)(s - j->s_base);
      if (j->dist_sum) j->dist_sum[row] = ds;
      j->unreachable += (int64_t)(N - 1) - reached;
      if (j->dist_out) memcpy(j->dist_out + row * (size_t)N, sc.dist, sizeof(int32_t) * (size_t)N);
      if (j->sigma_out) memcpy(j->sigma_out + row * (size_t)N, sc.sigma, sizeof(uint64_t) * (size_t)N);
    }
  }
  free(sc.dist);
  free(sc.sigma);
  free(sc.delta);
  free(sc.order);
  return NULL;
}

/*
 * Sources src_begin .. src_begin+src_count-1 of the topology given as an
 * out-neighbour CSR.  Outputs (each may be NULL): dist_out / sigma_out are
 * [src_count][N]; load is [E] and is overwritten with the sum over these sources;
 * dist_sum is [src_count]; *unreachable counts ordered pairs (s,t), t != s, with
 * no path; *flags bit0 = some sigma >= 2^53, bit1 = some pair unreachable.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int a2a_oracle_run(int32_t N, const int32_t* row_ptr, const int32_t* col, int32_t src_begin,
                   int32_t src_count, int32_t threads, int32_t* dist_out, uint64_t* sigma_out,
                   double* load, int64_t* dist_sum, int64_t* unreachable, int64_t* flags) {
  if (N <= 0 || !row_ptr || src_begin < 0 || src_count < 0 || src_begin + (int64_t)src_count > N)
    return -1;
  int64_t E = row_ptr[N];
  if (E > 0 && !col) return -1;
  if (threads < 1) threads = 1;
  if (threads > src_count) threads = src_count > 0 ? src_count : 1;
  job* jobs = (job*)calloc((size_t)threads, sizeof(job));
  pthread_t* tid = (pthread_t*)calloc((size_t)threads, sizeof(pthread_t));
  if (!jobs || !tid) return -1;
  int rc = 0;
  for (int t = 0; t < threads; ++t) {
    job* j = &jobs[t];
    j->N = N;
    j->row_ptr = row_ptr;
    j->col = col;
    j->s_base = src_begin;
    j->s_begin = src_begin + (int32_t)(((int64_t)src_count * t) / threads);
    j->s_end = src_begin + (int32_t)(((int64_t)src_count * (t + 1)) / threads);
    j->dist_out = dist_out;
    j->sigma_out = sigma_out;
    j->dist_sum = dist_sum;
    if (load) {
      j->load = (double*)calloc((size_t)(E > 0 ? E : 1), sizeof(double));
      if (!j->load) rc = -1;
    }
  }
  if (rc == 0) {
    for (int t = 1; t < threads; ++t) pthread_create(&tid[t], NULL, worker, &jobs[t]);
    worker(&jobs[0]);
    for (int t = 1; t < threads; ++t) pthread_join(tid[t], NULL);
  }
  int64_t unr = 0, fl = 0;
  if (load) memset(load, 0, sizeof(double) * (size_t)E);
  for (int t = 0; t < threads; ++t) {
    if (jobs[t].failed) rc = -1;
    unr += jobs[t].unreachable;
    if (jobs[t].overflow) fl |= 1;
    if (load && jobs[t].load)
      for (int64_t a = 0; a < E; ++a) load[a] += jobs[t].load[a];
    free(jobs[t].load);
  }
  if (unr) fl |= 2;
  if (unreachable) *unreachable = unr;
  if (flags) *flags = fl;
  free(jobs);
  free(tid);
  return rc;
}

/*
 * Link loads for commodities of unequal demand.  The paper's commodities all have the same
 * demand (Sec. 3.1.1); here commodity (s,t) carries demand[(s - src_begin) * N + t] >= 0, split
 * equally over its shortest paths as before (Sec. 5.2), so that
 *   load[a] = sum_{s,t != s} demand(s,t) * (#shortest s->t paths through a) / sigma(s,t).
 * In the dependency recursion the demand takes the place of the unit that every target
 * contributes: the traffic over link (u,w) on behalf of source s is
 * sigma(s,u)/sigma(s,w) * (demand(s,w) + delta(s,w)).  demand(s,s) and the demand of pairs
 * without a path are ignored.  *weighted_dist = sum_{s,t} demand(s,t) * D(s,t) over reachable
 * pairs, the link-time the demands need at least (the quantity that replaces sum D in the
 * capacity argument of Theorem 1).  Serial, sources in ascending order.
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int a2a_oracle_run_demand(int32_t N, const int32_t* row_ptr, const int32_t* col, int32_t src_begin,
                          int32_t src_count, const double* demand, double* load,
                          double* weighted_dist) {
  if (N <= 0 || !row_ptr || !demand || !load || src_begin < 0 || src_count < 0 ||
      src_begin + (int64_t)src_count > N)
    return -1;
  int64_t E = row_ptr[N];
  if (E > 0 && !col) return -1;
  src_scratch sc;
  sc.dist = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  sc.sigma = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)N);
  sc.delta = (double*)malloc(sizeof(double) * (size_t)N);
  sc.order = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  int rc = (!sc.dist || !sc.sigma || !sc.delta || !sc.order) ? -1 : 0;
  double wd = 0.0;
  if (rc == 0) {
    memset(load, 0, sizeof(double) * (size_t)E);
    for (int32_t s = src_begin; s < src_begin + src_count; ++s) {
      const double* dem = demand + (size_t)(s - src_begin) * (size_t)N;
      int64_t reached = 0;
      int overflow = 0;
      /* distances, path counts and the BFS order; no loads yet */
      (void)one_source(N, row_ptr, col, s, &sc, NULL, &reached, &overflow);
      for (int32_t i = (int32_t)reached; i >= 0; --i) {
        int32_t u = sc.order[i];
        if (u != s) wd += dem[u] * (double)sc.dist[u];
        for (int32_t a = row_ptr[u]; a < row_ptr[u + 1]; ++a) {
          int32_t w = col[a];
          if (sc.dist[w] == sc.dist[u] + 1) {
            double c = (double)sc.sigma[u] / (double)sc.sigma[w] * (dem[w] + sc.delta[w]);
            load[a] += c;
            sc.delta[u] += c;
          }
        }
      }
    }
  }
  if (weighted_dist) *weighted_dist = wd;
  free(sc.dist);
  free(sc.sigma);
  free(sc.delta);
  free(sc.order);
  return rc;
}

/*
 * Single-path baseline "SSSP" (Sec. 5.2): a heuristic that computes shortest paths iteration by
 * iteration through a graph whose link weights reflect the congestion that the earlier
 * iterations have caused; every commodity gets ONE path.  The paper gives neither the weights
 * nor what an iteration is; the reading taken here (parity unpinned against the paper, pinned
 * by the invariants and the path enumeration of tests/test_sssp.py):
 *   - an iteration routes the commodities of `iter_sources` consecutive sources (1 = source by
 *     source, the classic form of the heuristic) against the weights it starts with;
 *   - the weight of link a in an iteration is W[a] = number of commodities that the earlier
 *     iterations routed over a (0 for all links in the first one);
 *   - the path of commodity (s,t) is a path of D(s,t) links (hop count comes first: the baseline
 *     is a shortest-path scheme like EwSP), among those one of least total weight, among those
 *     the one whose last link has the lowest id, then the one before it, and so on; this is
 *     what the recursion cost(s,w) = min over links a=(u,w) with D(s,u)+1 = D(s,w) of
 *     cost(s,u) + W[a], ties to the lowest a, computes, and the paths of one source form a tree;
 *   - after the iteration every link's load grows by the number of paths of the iteration over it.
 * load[a] (int64, overwritten) = number of the commodities with source in
 * src_begin .. src_begin+src_count-1 routed over a; iterations take the sources in ascending
 * order.  dist_sum (may be NULL): [src_count] sum_t D(s,t); *unreachable (may be NULL): pairs
 * without a path (they are not routed).  Serial.  Returns 0, or -1 on bad arguments /
 * allocation failure.
 */
int a2a_oracle_sssp(int32_t N, const int32_t* row_ptr, const int32_t* col, int32_t src_begin,
                    int32_t src_count, int32_t iter_sources, int64_t* load, int64_t* dist_sum,
                    int64_t* unreachable) {
  if (N <= 0 || !row_ptr || !load || src_begin < 0 || src_count < 0 || iter_sources < 1 ||
      src_begin + (int64_t)src_count > N)
    return -1;
  int64_t E = row_ptr[N];
  if (E > 0 && !col) return -1;
  size_t En = (size_t)(E > 0 ? E : 1);
  int32_t* dist = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  int32_t* order = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  int64_t* cost = (int64_t*)malloc(sizeof(int64_t) * (size_t)N);
  int64_t* pred = (int64_t*)malloc(sizeof(int64_t) * (size_t)N); /* link id into the node, -1 none */
  int64_t* sub = (int64_t*)malloc(sizeof(int64_t) * (size_t)N);  /* paths that end in or pass the node */
  int32_t* tail = (int32_t*)malloc(sizeof(int32_t) * En);        /* node a link leaves from */
  int64_t* weight = (int64_t*)malloc(sizeof(int64_t) * En);
  int rc = (!dist || !order || !cost || !pred || !sub || !tail || !weight) ? -1 : 0;
  int64_t unr = 0;
  if (rc == 0) {
    for (int32_t u = 0; u < N; ++u)
      for (int32_t a = row_ptr[u]; a < row_ptr[u + 1]; ++a) tail[a] = u;
    memset(load, 0, sizeof(int64_t) * (size_t)E);
    for (int32_t s0 = src_begin; s0 < src_begin + src_count; s0 += iter_sources) {
      int32_t s1 = s0 + iter_sources;
      if (s1 > src_begin + src_count) s1 = src_begin + src_count;
      memcpy(weight, load, sizeof(int64_t) * (size_t)E); /* what the earlier iterations left */
      for (int32_t s = s0; s < s1; ++s) {
        int32_t head = 0, tl = 0;
        int64_t ds = 0;
        for (int32_t v = 0; v < N; ++v) {
          dist[v] = -1;
          pred[v] = -1;
          cost[v] = 0;
          sub[v] = 1;
        }
        dist[s] = 0;
        order[tl++] = s;
        while (head < tl) { /* FIFO order = level order: cost[u] is final when u is taken out */
          int32_t u = order[head++];
          for (int32_t a = row_ptr[u]; a < row_ptr[u + 1]; ++a) {
            int32_t w = col[a];
            if (dist[w] < 0) {
              dist[w] = dist[u] + 1;
              ds += dist[w];
              order[tl++] = w;
            }
            if (dist[w] == dist[u] + 1) {
              int64_t c = cost[u] + weight[a];
              if (pred[w] < 0 || c < cost[w] || (c == cost[w] && a < pred[w])) {
                cost[w] = c;
                pred[w] = a;
              }
            }
          }
        }
        for (int32_t i = tl - 1; i >= 1; --i) { /* deepest first: sub[w] is final when w is met */
          int32_t w = order[i];
          load[pred[w]] += sub[w];
          sub[tail[pred[w]]] += sub[w];
        }
        if (dist_sum) dist_sum[s - src_begin] = ds;
        unr += (int64_t)N - tl;
      }
    }
  }
  if (unreachable) *unreachable = unr;
  free(dist);
  free(order);
  free(cost);
  free(pred);
  free(sub);
  free(tail);
  free(weight);
  return rc;
}

/*
 * Schedule figures from the link loads.  out[] (10 doubles):
 *  0 max link load Lmax          (all-to-all time under unit demand/capacity, Sec. 5.3)
 *  1 lowest link id attaining it
 *  2 min link load
 *  3 t_sched   = Lmax * m / b
 *  4 t_lb_nd   = sumD * m / (N * dmax * b)   (Eq. (lb): demand sum D against capacity N d)
 *  5 t_lb_links= sumD * m / (E * b)          (same argument with the true link count)
 *  6 ratio     = t_sched / t_lb_nd
 *  7 throughput= (N-1) m / t_sched           (Sec. 2.2)
 *  8 f         = 1 / Lmax                    (concurrent flow value the loads realise)
 *  9 upper     = (N-1) f b                   (Sec. 5.1)
 */
int a2a_oracle_bound(int32_t N, const int32_t* row_ptr, const double* load, int64_t sum_dist,
                     double m, double b, double* out) {
  if (N <= 0 || !row_ptr || !out) return -1;
  int64_t E = row_ptr[N];
  if (E <= 0 || !load) return -1;
  int32_t dmax = 0;
  for (int32_t u = 0; u < N; ++u)
    if (row_ptr[u + 1] - row_ptr[u] > dmax) dmax = row_ptr[u + 1] - row_ptr[u];
  double lmax = load[0], lmin = load[0];
  int64_t arg = 0;
  for (int64_t a = 1; a < E; ++a) {
    if (load[a] > lmax) {
      lmax = load[a];
      arg = a;
    }
    if (load[a] < lmin) lmin = load[a];
  }
  out[0] = lmax;
  out[1] = (double)arg;
  out[2] = lmin;
  out[3] = lmax * m / b;
  out[4] = (double)sum_dist * m / ((double)N * (double)dmax * b);
  out[5] = (double)sum_dist * m / ((double)E * b);
  out[6] = out[3] / out[4];
  out[7] = (double)(N - 1) * m / out[3];
  out[8] = 1.0 / lmax;
  out[9] = (double)(N - 1) * out[8] * b;
  return 0;
}

/*
 * The same figures for a network G = (V, E, cap) with link capacities (Sec. 3.1.1): the flows of
 * a routing fit when every link's load, scaled by the common rate, stays within its capacity,
 * so the all-to-all time of the routing is the largest load / cap over the links (Sec. 5.3 with
 * unit capacities).  cap[a] multiplies the bandwidth b of a unit link.  out[] (12 doubles):
 *  0 max utilisation Umax = max_a load[a] / cap[a]
 *  1 lowest link id attaining it
 *  2 min utilisation
 *  3 t_sched    = Umax * m / b
 *  4 t_lb_nd    = sumD * m / (N * cmax * b), cmax = largest total out-capacity of a node
 *                 (Eq. (lb) with "d x N" read as the capacity N nodes of that out-capacity have)
 *  5 t_lb_links = sumD * m / (sum_a cap[a] * b)   (demand sum D against the true total capacity)
 *  6 ratio      = t_sched / t_lb_nd
 *  7 throughput = (N-1) m / t_sched
 *  8 f          = 1 / Umax
 *  9 upper      = (N-1) f b
 * 10 sum_a cap[a]
 * 11 cmax
 * Returns -2 if some capacity is not a positive finite number.
 */
int a2a_oracle_bound_cap(int32_t N, const int32_t* row_ptr, const double* load, const double* cap,
                         int64_t sum_dist, double m, double b, double* out) {
  if (N <= 0 || !row_ptr || !out) return -1;
  int64_t E = row_ptr[N];
  if (E <= 0 || !load || !cap) return -1;
  for (int64_t a = 0; a < E; ++a)
    if (!(cap[a] > 0.0) || cap[a] > 1.7976931348623157e308) return -2;
  double umax = load[0] / cap[0], umin = umax, total = 0.0, cmax = 0.0;
  int64_t arg = 0;
  for (int32_t u = 0; u < N; ++u) {
    double node_cap = 0.0;
    for (int32_t a = row_ptr[u]; a < row_ptr[u + 1]; ++a) {
      double util = load[a] / cap[a];
      if (util > umax) {
        umax = util;
        arg = a;
      }
      if (util < umin) umin = util;
      node_cap += cap[a];
      total += cap[a];
    }
    if (node_cap > cmax) cmax = node_cap;
  }
  out[0] = umax;
  out[1] = (double)arg;
  out[2] = umin;
  out[3] = umax * m / b;
  out[4] = (double)sum_dist * m / ((double)N * cmax * b);
  out[5] = (double)sum_dist * m / (total * b);
  out[6] = out[3] / out[4];
  out[7] = (double)(N - 1) * m / out[3];
  out[8] = 1.0 / umax;
  out[9] = (double)(N - 1) * out[8] * b;
  out[10] = total;
  out[11] = cmax;
  return 0;
}

/*
 * Distance sum of the fullest d-ary arborescence on N nodes (proof of Theorem 1, Sec. 5.4): the
 * tree whose level l holds d^l nodes until all N are placed.  Written out as the definition on
 * heap numbering: node 0 is the root, the parent of node i > 0 is (i-1)/d, and the level of a
 * node is one more than its parent's.  O(N) memory; test sizes only.
 */
int64_t a2a_oracle_tree_sum(int32_t N, int32_t d) {
  if (N < 1 || d < 1) return -1;
  int32_t* level = (int32_t*)malloc(sizeof(int32_t) * (size_t)N);
  if (!level) return -1;
  int64_t sum = 0;
  level[0] = 0;
  for (int32_t i = 1; i < N; ++i) {
    level[i] = level[(i - 1) / d] + 1;
    sum += level[i];
  }
  free(level);
  return sum;
}
