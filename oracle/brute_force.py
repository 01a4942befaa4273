"""Second oracle for tiny graphs: enumerate every shortest path, exact rationals.

Test infrastructure only.  Follows the plain definition of the EwSP scheme
(Sec. 5.2): each ordered pair (s,t) sends one unit, split equally over all of
its shortest link sequences.  Nothing is shared with a2a_oracle.c: distances come
from exhaustive relaxation (Bellman-Ford style, no queue), paths from depth-first
enumeration of all walks of exactly D(s,t) links, and the split is a Fraction.
Exponential: use for N <= 12 only.
"""
from __future__ import annotations

from fractions import Fraction
from typing import Dict, List, Tuple


def distances_by_relaxation(row_ptr, col_idx) -> List[List[int]]:
    """All-pairs hop counts by repeated relaxation over every link; -1 = no path."""
    N = len(row_ptr) - 1
    INF = 10 ** 9
    D = [[0 if i == j else INF for j in range(N)] for i in range(N)]
    for s in range(N):
        changed = True
        while changed:
            changed = False
            for u in range(N):
                if D[s][u] >= INF:
                    continue
                for a in range(row_ptr[u], row_ptr[u + 1]):
                    w = int(col_idx[a])
                    if D[s][u] + 1 < D[s][w]:
                        D[s][w] = D[s][u] + 1
                        changed = True
    return [[-1 if x >= INF else x for x in r] for r in D]


def shortest_paths(row_ptr, col_idx, D, s: int, t: int) -> List[Tuple[int, ...]]:
    """Every link sequence (tuple of link ids) from s to t of length D[s][t]."""
    out: List[Tuple[int, ...]] = []
    L = D[s][t]
    if L <= 0:
        return out

    def walk(u: int, used: Tuple[int, ...]):
        if len(used) == L:
            if u == t:
                out.append(used)
            return
        for a in range(row_ptr[u], row_ptr[u + 1]):
            walk(int(col_idx[a]), used + (a,))

    walk(s, ())
    return out


def ewsp(row_ptr, col_idx):
    """Returns (D, sigma, load) with load[a] a Fraction, and per-commodity link flows.

    per_commodity[(s,t)] maps link id -> Fraction carried for that pair.
    """
    row_ptr = [int(x) for x in row_ptr]
    col_idx = [int(x) for x in col_idx]
    N = len(row_ptr) - 1
    E = row_ptr[-1]
    D = distances_by_relaxation(row_ptr, col_idx)
    sigma = [[0] * N for _ in range(N)]
    load = [Fraction(0)] * E
    per_commodity: Dict[Tuple[int, int], Dict[int, Fraction]] = {}
    for s in range(N):
        sigma[s][s] = 1
        for t in range(N):
            if t == s or D[s][t] < 0:
                continue
            paths = shortest_paths(row_ptr, col_idx, D, s, t)
            sigma[s][t] = len(paths)
            share = Fraction(1, len(paths))
            flows: Dict[int, Fraction] = {}
            for p in paths:
                for a in p:
                    flows[a] = flows.get(a, Fraction(0)) + share
            per_commodity[(s, t)] = flows
            for a, f in flows.items():
                load[a] = load[a] + f
    return D, sigma, load, per_commodity


def sssp(row_ptr, col_idx, iter_sources: int = 1, src_begin: int = 0, src_count=None):
    """Single-path SSSP baseline (Sec. 5.2) by enumeration: returns (load, chosen) with load[a] the number
    of commodities routed over link a and chosen[(s,t)] the link sequence picked for the pair.

    Iterations take `iter_sources` consecutive sources; within one, the weight of a link is the number of
    commodities routed over it by the earlier iterations.  For every pair all link sequences of D(s,t) links
    are written out and the one of least total weight is taken; among equals the one with the lowest last
    link id, then the lowest link before it, and so on (the sequences are compared back to front)."""
    row_ptr = [int(x) for x in row_ptr]
    col_idx = [int(x) for x in col_idx]
    N = len(row_ptr) - 1
    if src_count is None:
        src_count = N - src_begin
    D = distances_by_relaxation(row_ptr, col_idx)
    load = [0] * row_ptr[-1]
    chosen: Dict[Tuple[int, int], Tuple[int, ...]] = {}
    for s0 in range(src_begin, src_begin + src_count, iter_sources):
        weight = list(load)
        for s in range(s0, min(s0 + iter_sources, src_begin + src_count)):
            for t in range(N):
                if t == s or D[s][t] < 0:
                    continue
                paths = shortest_paths(row_ptr, col_idx, D, s, t)
                best = min(paths, key=lambda p: (sum(weight[a] for a in p), tuple(reversed(p))))
                chosen[(s, t)] = best
                for a in best:
                    load[a] += 1
    return load, chosen
