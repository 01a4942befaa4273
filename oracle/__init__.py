"""CPU oracle (test infrastructure).

Only tests/, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg may
import this package.  It never imports the HIP library or its binding.

``a2a_oracle.c`` is the serial BFS + dependency-accumulation oracle (built with
gcc into ``liba2a_oracle.so`` by :func:`build`); ``brute_force.py`` is the second,
exact-rational oracle for tiny graphs (enumerates every shortest path).
"""
from .binding import (  # noqa: F401
    build,
    run,
    run_demand,
    bound,
    bound_cap,
    tree_sum,
    sssp,
    OracleResult,
    BOUND_FIELDS,
    CAP_FIELDS,
)
