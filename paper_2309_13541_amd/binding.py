"""ctypes binding of liba2a_topo.so: same names as include/a2a_topo.h, marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams, nothing
else); their ``data_ptr()`` and the current stream's handle cross the C ABI as plain pointers.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_SRC = os.path.join(_HERE, "csrc", "a2a_topo.hip")
_LIB = os.path.join(_HERE, "liba2a_topo.so")
_lib = None

OK = 0
ERR_INVALID_ARG = -1
ERR_SELF_LOOP = -2
ERR_WORKSPACE_TOO_SMALL = -3
ERR_HIP = -4
ERR_NOT_IMPLEMENTED = -5
ERR_DISCONNECTED = -6
ERR_NO_MEMORY = -7
ERR_LEVEL_OVERFLOW = -8

WS_DISTANCES = 0x0
WS_SIGMA = 0x1
WS_LOADS = 0x2
WS_SSSP = 0x4
WS_MINIMAL = 0x100
FLAG_SIGMA_INEXACT = 0x1
FLAG_UNREACHABLE = 0x2

EXPORTED_SYMBOLS = (
    "a2a_topo_create", "a2a_topo_destroy", "a2a_topo_info", "a2a_workspace_bytes",
    "a2a_distances", "a2a_link_loads", "a2a_link_loads_demand", "a2a_schedule_bound", "a2a_status_string",
    "a2a_profile_enable", "a2a_profile_read", "a2a_tree_lower_bound", "a2a_schedule_bound_cap",
    "a2a_link_loads_static", "a2a_sssp_loads",
)
STATIC_WORKSPACE_BYTES = 32 << 20

PROF_KERNELS = ("init", "bfs", "offsets", "fwd_rows", "fwd_few", "fwd_spread", "bwd_rows", "bwd_few", "bwd_spread",
                "reduce", "extract")
PROF_MAX_LEVELS = 64

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


class A2AError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


class Bound(ctypes.Structure):
    """Mirror of ``a2a_bound``."""
    _fields_ = [
        ("max_load", ctypes.c_double), ("argmax_arc", ctypes.c_int64), ("min_load", ctypes.c_double),
        ("sum_dist", ctypes.c_int64), ("n_links", ctypes.c_int64), ("n_nodes", ctypes.c_int32),
        ("dmax", ctypes.c_int32), ("t_sched", ctypes.c_double), ("t_lb_nd", ctypes.c_double),
        ("t_lb_links", ctypes.c_double), ("ratio", ctypes.c_double), ("throughput", ctypes.c_double),
        ("flow_value", ctypes.c_double), ("throughput_upper", ctypes.c_double),
    ]

    def as_dict(self) -> dict:
        return {n: getattr(self, n) for n, _ in self._fields_}


class BoundCap(ctypes.Structure):
    """Mirror of ``a2a_bound_cap``."""
    _fields_ = [
        ("max_util", ctypes.c_double), ("argmax_arc", ctypes.c_int64), ("min_util", ctypes.c_double),
        ("sum_dist", ctypes.c_int64), ("n_links", ctypes.c_int64), ("n_nodes", ctypes.c_int32),
        ("reserved", ctypes.c_int32), ("total_capacity", ctypes.c_double),
        ("max_node_capacity", ctypes.c_double), ("t_sched", ctypes.c_double), ("t_lb_nd", ctypes.c_double),
        ("t_lb_links", ctypes.c_double), ("ratio", ctypes.c_double), ("throughput", ctypes.c_double),
        ("flow_value", ctypes.c_double), ("throughput_upper", ctypes.c_double),
    ]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_ if n != "reserved"}


class TreeBound(ctypes.Structure):
    """Mirror of ``a2a_tree_bound``."""
    _fields_ = [("s_min", ctypes.c_int64), ("height", ctypes.c_int32), ("full", ctypes.c_int32),
                ("t_lb", ctypes.c_double), ("throughput_ub", ctypes.c_double)]


class Profile(ctypes.Structure):
    """Mirror of ``a2a_profile``."""
    _fields_ = [("ms", ctypes.c_double * 16), ("launches", ctypes.c_int64 * 16),
                ("ms_level", (ctypes.c_double * PROF_MAX_LEVELS) * 16),
                ("pairs_level", ctypes.c_int64 * PROF_MAX_LEVELS),
                ("dag_level", ctypes.c_int64 * PROF_MAX_LEVELS),
                ("dag_links", ctypes.c_int64), ("calls", ctypes.c_int64),
                ("depth", ctypes.c_int32), ("groups", ctypes.c_int32), ("narrow_levels", ctypes.c_uint64),
                ("fwd_flavours", ctypes.c_uint64), ("bwd_flavours", ctypes.c_uint64)]

    def as_dict(self) -> dict:
        d = {"dag_links": self.dag_links, "calls": self.calls, "depth": self.depth,
             "groups": self.groups, "narrow_levels": self.narrow_levels, "fwd_flavours": self.fwd_flavours,
             "bwd_flavours": self.bwd_flavours, "pairs_level": list(self.pairs_level),
             "dag_level": list(self.dag_level)}
        for i, n in enumerate(PROF_KERNELS):
            d[n] = {"ms": self.ms[i], "launches": self.launches[i], "ms_level": list(self.ms_level[i])}
        return d


def library_path() -> str:
    return _LIB


def build_library(verbose: bool = False) -> str:
    """Compile csrc/a2a_topo.hip for gfx950 with hipcc (works without a GPU)."""
    global _lib
    cmd = ["hipcc", *HIPCC_FLAGS, "-I" + os.path.join(_ROOT, "include"), "-o", _LIB, _SRC]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    _lib = None
    return _LIB


def load_library():
    """Load liba2a_topo.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        raise RuntimeError(
            f"{_LIB} is missing: build it with paper_2309_13541_amd.build_library() "
            "(or __graft_entry__.build()); there is no CPU fallback")
    # PyTorch ships its own HIP runtime (same soname as the system one).  It has to be in the
    # process first, so that this library binds to the runtime that owns torch's tensors and
    # streams instead of bringing in a second one.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.a2a_topo_create.restype = ctypes.c_int
    lib.a2a_topo_create.argtypes = [i32, vp, vp, ctypes.POINTER(vp)]
    lib.a2a_topo_destroy.restype = None
    lib.a2a_topo_destroy.argtypes = [vp]
    lib.a2a_topo_info.restype = ctypes.c_int
    lib.a2a_topo_info.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i64), ctypes.POINTER(i32),
                                  ctypes.POINTER(i32)]
    lib.a2a_workspace_bytes.restype = sz
    lib.a2a_workspace_bytes.argtypes = [vp, i32, ctypes.c_int]
    lib.a2a_distances.restype = ctypes.c_int
    lib.a2a_distances.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.a2a_link_loads.restype = ctypes.c_int
    lib.a2a_link_loads.argtypes = [vp, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.a2a_link_loads_static.restype = ctypes.c_int
    lib.a2a_link_loads_static.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    lib.a2a_sssp_loads.restype = ctypes.c_int
    lib.a2a_sssp_loads.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.a2a_link_loads_demand.restype = ctypes.c_int
    lib.a2a_link_loads_demand.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.a2a_schedule_bound_cap.restype = ctypes.c_int
    lib.a2a_schedule_bound_cap.argtypes = [vp, vp, vp, i64, i64, ctypes.c_double, ctypes.c_double, vp, vp]
    lib.a2a_schedule_bound.restype = ctypes.c_int
    lib.a2a_schedule_bound.argtypes = [vp, vp, i64, i64, ctypes.c_double, ctypes.c_double,
                                       ctypes.POINTER(Bound), vp]
    lib.a2a_profile_enable.restype = ctypes.c_int
    lib.a2a_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.a2a_profile_read.restype = ctypes.c_int
    lib.a2a_profile_read.argtypes = [vp, ctypes.POINTER(Profile)]
    lib.a2a_tree_lower_bound.restype = ctypes.c_int
    lib.a2a_tree_lower_bound.argtypes = [i32, i32, ctypes.c_double, ctypes.c_double, ctypes.POINTER(TreeBound)]
    lib.a2a_status_string.restype = ctypes.c_char_p
    lib.a2a_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().a2a_status_string(int(status)).decode()


def tree_lower_bound(N: int, d: int, m_bytes: float = 1.0, b_bytes_per_s: float = 1.0) -> TreeBound:
    """a2a_tree_lower_bound: Theorem 1's bound for any N-host, degree-d topology (host arithmetic)."""
    out = TreeBound()
    _check(load_library().a2a_tree_lower_bound(int(N), int(d), float(m_bytes), float(b_bytes_per_s),
                                               ctypes.byref(out)), "a2a_tree_lower_bound")
    return out


def _check(status: int, where: str, allow=()):
    if status != OK and status not in allow:
        raise A2AError(status, where)
    return status


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


class Topology:
    """Owns an ``a2a_topo`` handle.  Methods are the C entry points with the same names."""

    def __init__(self, row_ptr, col_idx):
        lib = load_library()
        rp = np.ascontiguousarray(row_ptr, dtype=np.int32)
        ci = np.ascontiguousarray(col_idx, dtype=np.int32)
        h = ctypes.c_void_p()
        _check(lib.a2a_topo_create(len(rp) - 1, rp.ctypes.data, ci.ctypes.data if len(ci) else None,
                                   ctypes.byref(h)), "a2a_topo_create")
        self._h = h
        n, e, d, lb = ctypes.c_int32(), ctypes.c_int64(), ctypes.c_int32(), ctypes.c_int32()
        _check(lib.a2a_topo_info(h, ctypes.byref(n), ctypes.byref(e), ctypes.byref(d), ctypes.byref(lb)),
               "a2a_topo_info")
        self.N, self.E, self.dmax, self.level_bound = n.value, e.value, d.value, lb.value

    def close(self):
        if getattr(self, "_h", None):
            load_library().a2a_topo_destroy(self._h)
            self._h = None

    __del__ = close

    def workspace_bytes(self, src_count: int, flags: int) -> int:
        return int(load_library().a2a_workspace_bytes(self._h, src_count, flags))

    def alloc_workspace(self, src_count: int, flags: int, max_bytes: Optional[int] = None):
        """A torch uint8 device tensor of the recommended size, capped at max_bytes."""
        import torch
        want = self.workspace_bytes(src_count, flags)
        least = self.workspace_bytes(src_count, flags | WS_MINIMAL)
        if max_bytes is not None:
            want = max(least, min(want, int(max_bytes)))
        return torch.empty(want, dtype=torch.uint8, device="cuda")

    def distances(self, src_begin: int, src_count: int, *, dist=None, sigma=None, dist_sum=None,
                  unreachable=None, flags=None, workspace, stream=None) -> int:
        return _check(load_library().a2a_distances(
            self._h, src_begin, src_count, _ptr(dist), _ptr(sigma), _ptr(dist_sum), _ptr(unreachable),
            _ptr(flags), _ptr(workspace), workspace.numel() if workspace is not None else 0,
            _stream(stream)), "a2a_distances")

    def link_loads(self, src_begin: int, src_count: int, *, load, dist_sum_total=None, flags=None,
                   workspace, stream=None) -> int:
        return _check(load_library().a2a_link_loads(
            self._h, src_begin, src_count, _ptr(load), _ptr(dist_sum_total), _ptr(flags),
            _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream(stream)),
            "a2a_link_loads")

    def link_loads_static(self, src_begin: int, src_count: int, *, load, dist_sum_total=None, flags=None,
                          stream=None) -> int:
        """a2a_link_loads on the library's fixed workspace array (no device allocation in the call)."""
        return _check(load_library().a2a_link_loads_static(
            self._h, src_begin, src_count, _ptr(load), _ptr(dist_sum_total), _ptr(flags), _stream(stream)),
            "a2a_link_loads_static")

    def sssp_loads(self, src_begin: int, src_count: int, iter_sources: int = 64, *, load, dist_sum_total=None,
                   flags=None, workspace, stream=None) -> int:
        """a2a_sssp_loads: single-path SSSP baseline, one iteration per ``iter_sources`` sources."""
        return _check(load_library().a2a_sssp_loads(
            self._h, src_begin, src_count, iter_sources, _ptr(load), _ptr(dist_sum_total), _ptr(flags),
            _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream(stream)),
            "a2a_sssp_loads")

    def link_loads_demand(self, src_begin: int, src_count: int, *, demand, load, weighted_dist=None,
                          dist_sum_total=None, flags=None, workspace, stream=None) -> int:
        """``demand``: device float64 [N][src_count], ``demand[t][s - src_begin]`` = what s sends to t."""
        return _check(load_library().a2a_link_loads_demand(
            self._h, src_begin, src_count, _ptr(demand), _ptr(load), _ptr(weighted_dist), _ptr(dist_sum_total),
            _ptr(flags), _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream(stream)),
            "a2a_link_loads_demand")

    def profile_enable(self, mode: int = 1) -> None:
        """0 off, 1 per-launch events, 2 events + count of shortest-path (source, link) pairs."""
        _check(load_library().a2a_profile_enable(self._h, int(mode)), "a2a_profile_enable")

    def profile_read(self) -> dict:
        out = Profile()
        _check(load_library().a2a_profile_read(self._h, ctypes.byref(out)), "a2a_profile_read")
        return out.as_dict()

    def schedule_bound(self, load, sum_dist: int, flags: int = 0, m_bytes: float = 1.0,
                       b_bytes_per_s: float = 1.0, stream=None, allow_disconnected: bool = False):
        out = Bound()
        st = load_library().a2a_schedule_bound(self._h, _ptr(load), int(sum_dist), int(flags),
                                               float(m_bytes), float(b_bytes_per_s), ctypes.byref(out),
                                               _stream(stream))
        _check(st, "a2a_schedule_bound", allow=(ERR_DISCONNECTED,) if allow_disconnected else ())
        return out, st

    def schedule_bound_cap(self, load, cap, sum_dist: int, flags: int = 0, m_bytes: float = 1.0,
                           b_bytes_per_s: float = 1.0, stream=None, allow_disconnected: bool = False):
        out = BoundCap()
        st = load_library().a2a_schedule_bound_cap(self._h, _ptr(load), _ptr(cap), int(sum_dist), int(flags),
                                                   float(m_bytes), float(b_bytes_per_s), ctypes.byref(out),
                                                   _stream(stream))
        _check(st, "a2a_schedule_bound_cap", allow=(ERR_DISCONNECTED,) if allow_disconnected else ())
        return out, st
