"""Seeded synthetic topology generators (inputs only).

Every function returns a direct-connect topology as an int32 out-neighbour CSR
``(row_ptr[N+1], col_idx[E])``; CSR position = link id.  The families are the
ones the paper evaluates on (tori, hypercube, complete bipartite, generalized
Kautz, random regular: Sec. 5 "Testbed", Sec. 5.4) plus tiny hand-made graphs
for edge cases.  This module holds no BFS, path counting or load arithmetic:
it is shared by the CPU oracle's tests and the GPU library's tests, which share
nothing else.
"""
from .topologies import (  # noqa: F401
    csr_from_rows,
    torus,
    hypercube,
    imase_itoh,
    random_regular,
    complete_bipartite,
    ring,
    bidirectional_ring,
    remove_arcs,
    remove_nodes,
    named_config,
    CONFIG_NAMES,
    lcg_stream,
)
