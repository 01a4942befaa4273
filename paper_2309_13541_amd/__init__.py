"""MI355X-native all-to-all topology evaluator (distances, path counts, EwSP link loads).

Thin Python layer over the C-ABI library ``liba2a_topo.so`` (built from ``csrc/`` by
:func:`build_library`); every step of the computation runs in HIP kernels.  Importing this
package does not load the library; the first call does, and fails loudly if it is missing.
"""
from .binding import (  # noqa: F401
    A2AError,
    Bound,
    BoundCap,
    Profile,
    PROF_KERNELS,
    Topology,
    TreeBound,
    tree_lower_bound,
    build_library,
    library_path,
    load_library,
    status_string,
    EXPORTED_SYMBOLS,
    STATIC_WORKSPACE_BYTES,
    WS_DISTANCES, WS_SIGMA, WS_LOADS, WS_SSSP, WS_MINIMAL,
    FLAG_SIGMA_INEXACT, FLAG_UNREACHABLE,
    OK, ERR_INVALID_ARG, ERR_SELF_LOOP, ERR_WORKSPACE_TOO_SMALL, ERR_HIP, ERR_NOT_IMPLEMENTED,
    ERR_DISCONNECTED, ERR_NO_MEMORY, ERR_LEVEL_OVERFLOW,
)
