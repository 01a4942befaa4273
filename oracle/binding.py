"""ctypes binding of the C oracle (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "a2a_oracle.c")
_LIB = os.path.join(_HERE, "liba2a_oracle.so")
_lib = None

BOUND_FIELDS = (
    "max_load", "argmax_arc", "min_load", "t_sched", "t_lb_nd", "t_lb_links",
    "ratio", "throughput", "flow_value", "throughput_upper",
)


def build(force: bool = True) -> str:
    """Compile the oracle with gcc -O2 (no SIMD intrinsics, no tuning)."""
    global _lib
    if force or not os.path.exists(_LIB):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra",
             "-o", _LIB, _SRC])
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build(force=True)
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.a2a_oracle_run.restype = ctypes.c_int
        lib.a2a_oracle_run.argtypes = [
            ctypes.c_int32, i32p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64)]
        lib.a2a_oracle_bound.restype = ctypes.c_int
        lib.a2a_oracle_bound.argtypes = [
            ctypes.c_int32, i32p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_double,
            ctypes.c_double, ctypes.c_void_p]
        lib.a2a_oracle_bound_cap.restype = ctypes.c_int
        lib.a2a_oracle_bound_cap.argtypes = [
            ctypes.c_int32, i32p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_double,
            ctypes.c_double, ctypes.c_void_p]
        lib.a2a_oracle_run_demand.restype = ctypes.c_int
        lib.a2a_oracle_run_demand.argtypes = [
            ctypes.c_int32, i32p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.POINTER(ctypes.c_double)]
        lib.a2a_oracle_sssp.restype = ctypes.c_int
        lib.a2a_oracle_sssp.argtypes = [
            ctypes.c_int32, i32p, i32p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64)]
        lib.a2a_oracle_tree_sum.restype = ctypes.c_int64
        lib.a2a_oracle_tree_sum.argtypes = [ctypes.c_int32, ctypes.c_int32]
        _lib = lib
    return _lib


@dataclass
class OracleResult:
    dist: Optional[np.ndarray]      # int32 [src_count, N], -1 = unreachable
    sigma: Optional[np.ndarray]     # uint64 [src_count, N]
    load: Optional[np.ndarray]      # float64 [E]
    dist_sum: np.ndarray            # int64 [src_count]
    unreachable: int
    flags: int
    threads: int


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def run(row_ptr, col_idx, src_begin: int = 0, src_count: Optional[int] = None, *,
        want_dist: bool = False, want_sigma: bool = False, want_load: bool = True,
        threads: int = 1) -> OracleResult:
    lib = _load()
    row_ptr, rp = _i32(row_ptr)
    col_idx, cp = _i32(col_idx)
    N = len(row_ptr) - 1
    E = int(row_ptr[-1])
    if src_count is None:
        src_count = N - src_begin
    dist = np.empty((src_count, N), dtype=np.int32) if want_dist else None
    sigma = np.empty((src_count, N), dtype=np.uint64) if want_sigma else None
    load = np.empty(E, dtype=np.float64) if want_load else None
    dist_sum = np.zeros(src_count, dtype=np.int64)
    unr = ctypes.c_int64(0)
    fl = ctypes.c_int64(0)

    def ptr(a):
        return None if a is None else a.ctypes.data

    rc = lib.a2a_oracle_run(N, rp, cp, src_begin, src_count, threads, ptr(dist), ptr(sigma),
                            ptr(load), ptr(dist_sum), ctypes.byref(unr), ctypes.byref(fl))
    if rc != 0:
        raise ValueError("a2a_oracle_run rejected its arguments")
    used = max(1, min(threads, src_count))
    return OracleResult(dist, sigma, load, dist_sum, unr.value, fl.value, used)


def bound(row_ptr, load, sum_dist: int, m: float = 1.0, b: float = 1.0) -> dict:
    lib = _load()
    row_ptr, rp = _i32(row_ptr)
    load = np.ascontiguousarray(load, dtype=np.float64)
    out = np.zeros(len(BOUND_FIELDS), dtype=np.float64)
    rc = lib.a2a_oracle_bound(len(row_ptr) - 1, rp, load.ctypes.data, int(sum_dist),
                              float(m), float(b), out.ctypes.data)
    if rc != 0:
        raise ValueError("a2a_oracle_bound rejected its arguments")
    res = dict(zip(BOUND_FIELDS, out.tolist()))
    res["argmax_arc"] = int(res["argmax_arc"])
    return res


CAP_FIELDS = BOUND_FIELDS + ("total_capacity", "max_node_capacity")


def bound_cap(row_ptr, load, cap, sum_dist: int, m: float = 1.0, b: float = 1.0) -> dict:
    """Schedule figures with link capacities; ValueError for a capacity that is not positive."""
    lib = _load()
    row_ptr, rp = _i32(row_ptr)
    load = np.ascontiguousarray(load, dtype=np.float64)
    cap = np.ascontiguousarray(cap, dtype=np.float64)
    if len(cap) != len(load):
        raise ValueError("cap and load differ in length")
    out = np.zeros(len(CAP_FIELDS), dtype=np.float64)
    rc = lib.a2a_oracle_bound_cap(len(row_ptr) - 1, rp, load.ctypes.data, cap.ctypes.data, int(sum_dist),
                                  float(m), float(b), out.ctypes.data)
    if rc != 0:
        raise ValueError("a2a_oracle_bound_cap rejected its arguments (%d)" % rc)
    res = dict(zip(CAP_FIELDS, out.tolist()))
    res["argmax_arc"] = int(res["argmax_arc"])
    return res


def tree_sum(N: int, d: int) -> int:
    """Distance sum of the fullest d-ary arborescence on N nodes (Theorem 1's proof)."""
    v = int(_load().a2a_oracle_tree_sum(int(N), int(d)))
    if v < 0:
        raise ValueError("a2a_oracle_tree_sum rejected its arguments")
    return v


def run_demand(row_ptr, col_idx, demand, src_begin: int = 0):
    """Link loads and demand-weighted distance sum for demand[s - src_begin][t] (one row per source)."""
    lib = _load()
    row_ptr, rp = _i32(row_ptr)
    col_idx, cp = _i32(col_idx)
    N = len(row_ptr) - 1
    demand = np.ascontiguousarray(demand, dtype=np.float64)
    if demand.ndim != 2 or demand.shape[1] != N:
        raise ValueError("demand must be [src_count][N]")
    load = np.empty(int(row_ptr[-1]), dtype=np.float64)
    wd = ctypes.c_double(0.0)
    rc = lib.a2a_oracle_run_demand(N, rp, cp, int(src_begin), int(demand.shape[0]), demand.ctypes.data,
                                   load.ctypes.data, ctypes.byref(wd))
    if rc != 0:
        raise ValueError("a2a_oracle_run_demand rejected its arguments")
    return load, wd.value


def sssp(row_ptr, col_idx, src_begin: int = 0, src_count: Optional[int] = None, iter_sources: int = 1):
    """Single-path SSSP baseline: (load int64[E], dist_sum int64[src_count], unreachable pairs)."""
    lib = _load()
    row_ptr, rp = _i32(row_ptr)
    col_idx, cp = _i32(col_idx)
    N = len(row_ptr) - 1
    if src_count is None:
        src_count = N - src_begin
    load = np.zeros(int(row_ptr[-1]), dtype=np.int64)
    dist_sum = np.zeros(src_count, dtype=np.int64)
    unr = ctypes.c_int64(0)
    rc = lib.a2a_oracle_sssp(N, rp, cp, int(src_begin), int(src_count), int(iter_sources), load.ctypes.data,
                             dist_sum.ctypes.data, ctypes.byref(unr))
    if rc != 0:
        raise ValueError("a2a_oracle_sssp rejected its arguments")
    return load, dist_sum, unr.value
