"""Shared test helpers: fixture parsing and tiny hand-made graphs (inputs only)."""
import os
from fractions import Fraction

from a2a_inputs import csr_from_rows

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def paper_values():
    out = {}
    with open(os.path.join(GOLDEN, "paper_values.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = [x.strip() for x in line.split("=", 1)]
            out[k] = v
    return out


def frac(s: str) -> Fraction:
    return Fraction(s.replace(" ", ""))


# s=0, a=1, b=2, c=3, d=4, t=5: three shortest 0->5 paths, two of them through node 1.
# Splitting per path puts 2/3 of commodity (0,5) on link 0->1; splitting per next
# hop would put 1/2 there.
ASYMMETRIC_ROWS = [[1, 2], [3, 4], [4], [5], [5], []]


def tiny_graphs():
    """name -> CSR, all with N <= 12."""
    from a2a_inputs import torus, hypercube, complete_bipartite, ring, remove_arcs
    g = {
        "cycle3": ring(3),
        "asymmetric_dag": csr_from_rows(ASYMMETRIC_ROWS),
        "k33": complete_bipartite(3),
        "k44": complete_bipartite(4),
        "torus3x4": torus([3, 4]),
        "cube3": hypercube(3),
        "torus2x2x2_parallel": torus([2, 2, 2]),
        # 0->1 twice (parallel links), 1->2, 2->0
        "parallel_path": csr_from_rows([[1, 1], [2], [0]]),
        # node 4 has no in-arcs and node 5 no arcs at all
        "unreachable": csr_from_rows([[1], [2], [0, 3], [0], [0], []]),
        "ring7_chord": csr_from_rows([[1, 3], [2], [3], [4], [5], [6], [0]]),
        "punctured_torus3x3": remove_arcs(torus([3, 3]), [0, 7, 20]),
    }
    return g
