"""Topology generators.  numpy only; no graph algorithms live here."""
from __future__ import annotations

import functools
from typing import Iterable, List, Sequence, Tuple

import numpy as np

CSR = Tuple[np.ndarray, np.ndarray]


def csr_from_rows(rows: Sequence[Iterable[int]]) -> CSR:
    """Pack per-node out-neighbour lists (order kept, duplicates kept)."""
    row_ptr = np.zeros(len(rows) + 1, dtype=np.int32)
    cols: List[int] = []
    for i, r in enumerate(rows):
        r = list(r)
        cols.extend(r)
        row_ptr[i + 1] = len(cols)
    return row_ptr, np.asarray(cols, dtype=np.int32).reshape(-1)


def torus(dims: Sequence[int]) -> CSR:
    """n-dimensional torus with wraparound, +-1 per dimension.

    Node id = x0 + k0*x1 + k0*k1*x2 ...; row order: dim 0 "+1", dim 0 "-1",
    dim 1 "+1", ...  A side of 2 yields two parallel arcs (kept as two links);
    a side of 1 would yield self-loops and is rejected.
    """
    dims = [int(k) for k in dims]
    if any(k < 2 for k in dims):
        raise ValueError("torus sides must be >= 2")
    n = int(np.prod(dims))
    ids = np.arange(n, dtype=np.int64)
    cols = np.empty((n, 2 * len(dims)), dtype=np.int64)
    stride = 1
    for a, k in enumerate(dims):
        x = (ids // stride) % k
        cols[:, 2 * a] = ids + (((x + 1) % k) - x) * stride
        cols[:, 2 * a + 1] = ids + (((x - 1) % k) - x) * stride
        stride *= k
    row_ptr = (np.arange(n + 1, dtype=np.int64) * (2 * len(dims))).astype(np.int32)
    return row_ptr, cols.reshape(-1).astype(np.int32)


def hypercube(n: int) -> CSR:
    """Binary n-cube: arc u -> u xor 2^k, row order k = 0..n-1."""
    N = 1 << n
    ids = np.arange(N, dtype=np.int64)[:, None]
    cols = ids ^ (1 << np.arange(n, dtype=np.int64))[None, :]
    row_ptr = (np.arange(N + 1, dtype=np.int64) * n).astype(np.int32)
    return row_ptr, cols.reshape(-1).astype(np.int32)


def imase_itoh(N: int, d: int) -> CSR:
    """Imase-Itoh generalized Kautz digraph: i -> (-d*i - j) mod N, j = 1..d.

    Non-negative residue, row order j = 1..d, self-loops dropped.
    """
    rows = []
    for i in range(N):
        rows.append([w for w in ((-d * i - j) % N for j in range(1, d + 1)) if w != i])
    return csr_from_rows(rows)


_LCG_MUL = 6364136223846793005
_LCG_INC = 1442695040888963407
_MASK64 = (1 << 64) - 1


def lcg_stream(seed: int):
    """64-bit LCG x <- x*6364136223846793005 + 1442695040888963407 (mod 2^64).

    Yields (x >> 11) after each advance; x0 = seed.
    """
    x = seed & _MASK64
    while True:
        x = (x * _LCG_MUL + _LCG_INC) & _MASK64
        yield x >> 11


def random_regular(N: int, d: int, seed: int) -> CSR:
    """Union of d uniform random permutations pi_0..pi_{d-1} of 0..N-1.

    One LCG stream (see lcg_stream) serves all permutations in order k = 0..d-1.
    Each permutation starts from the identity and is shuffled by Fisher-Yates:
    for i = N-1 .. 1: j = next() mod (i+1); swap(p[i], p[j]).  Row i lists
    pi_0(i) .. pi_{d-1}(i) in k order; self-loops are dropped, parallel arcs are
    kept as separate links.
    """
    gen = lcg_stream(seed)
    perms = []
    for _ in range(d):
        p = list(range(N))
        for i in range(N - 1, 0, -1):
            j = next(gen) % (i + 1)
            p[i], p[j] = p[j], p[i]
        perms.append(np.asarray(p, dtype=np.int64))
    P = np.stack(perms, axis=1)  # [N, d]
    keep = P != np.arange(N, dtype=np.int64)[:, None]
    row_ptr = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(keep.sum(axis=1), out=row_ptr[1:])
    return row_ptr.astype(np.int32), P[keep].astype(np.int32)


def complete_bipartite(k: int) -> CSR:
    """K_{k,k} as a digraph: node i < k -> k..2k-1, node i >= k -> 0..k-1."""
    rows = [list(range(k, 2 * k)) if i < k else list(range(k)) for i in range(2 * k)]
    return csr_from_rows(rows)


def ring(N: int) -> CSR:
    """Directed cycle i -> i+1 (mod N)."""
    return csr_from_rows([[(i + 1) % N] for i in range(N)])


def bidirectional_ring(N: int) -> CSR:
    """Cycle with arcs i -> i+1 and i -> i-1 (mod N)."""
    return torus([N])


def remove_arcs(csr: CSR, arc_ids: Iterable[int]) -> CSR:
    """Drop the links with the given CSR positions (a 'punctured' topology)."""
    row_ptr, col = csr
    E = int(row_ptr[-1])
    keep = np.ones(E, dtype=bool)
    keep[np.asarray(list(arc_ids), dtype=np.int64)] = False
    src = np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))
    new_ptr = np.zeros(len(row_ptr), dtype=np.int64)
    np.cumsum(np.bincount(src[keep], minlength=len(row_ptr) - 1), out=new_ptr[1:])
    return new_ptr.astype(np.int32), col[keep].astype(np.int32)


def remove_nodes(csr: CSR, nodes: Iterable[int]) -> CSR:
    """Delete nodes (and every arc touching them); survivors are renumbered in order."""
    row_ptr, col = csr
    N = len(row_ptr) - 1
    dead = np.zeros(N, dtype=bool)
    dead[np.asarray(list(nodes), dtype=np.int64)] = True
    new_id = np.cumsum(~dead) - 1
    rows = []
    for u in range(N):
        if dead[u]:
            continue
        rows.append([int(new_id[w]) for w in col[row_ptr[u]:row_ptr[u + 1]] if not dead[w]])
    return csr_from_rows(rows)


CONFIG_NAMES = ("C1", "C2", "C3", "C4", "C5")


@functools.lru_cache(maxsize=None)
def named_config(name: str) -> CSR:
    """The five benchmark topologies.

    C1 8x8 torus; C2 hypercube n=10; C3 16x16x16 torus; C4 Imase-Itoh N=16384 d=4;
    C5 random 8-regular N=65536 from seed 1234.
    """
    if name == "C1":
        return torus([8, 8])
    if name == "C2":
        return hypercube(10)
    if name == "C3":
        return torus([16, 16, 16])
    if name == "C4":
        return imase_itoh(16384, 4)
    if name == "C5":
        return random_regular(65536, 8, 1234)
    raise KeyError(name)
