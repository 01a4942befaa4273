"""C-ABI checks that need no GPU: the library loads, exports every declared symbol, and
validates its arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import a2a_inputs as gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def a2a():
    import paper_2309_13541_amd as lib
    if not os.path.exists(lib.library_path()):
        lib.build_library()
    lib.load_library()
    return lib


def declared_functions():
    text = open(os.path.join(ROOT, "include", "a2a_topo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(a2a_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(a2a):
    names = declared_functions()
    assert set(names) == set(a2a.EXPORTED_SYMBOLS)
    lib = ctypes.CDLL(a2a.library_path())
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(a2a):
    assert a2a.status_string(0) == "ok"
    seen = {a2a.status_string(s) for s in range(-8, 1)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert a2a.status_string(-99) == "unknown status"


def _create(a2a, N, rp, col):
    lib = a2a.load_library()
    h = ctypes.c_void_p()
    rp = np.ascontiguousarray(rp, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    st = lib.a2a_topo_create(N, rp.ctypes.data if len(rp) else None,
                             col.ctypes.data if len(col) else None, ctypes.byref(h))
    if st == 0:
        lib.a2a_topo_destroy(h)
    return st


def test_create_validates_before_any_device_call(a2a):
    rp, col = gen.torus([3, 3])
    assert _create(a2a, 0, rp, col) == a2a.ERR_INVALID_ARG
    assert _create(a2a, 9, [], col) == a2a.ERR_INVALID_ARG
    bad = rp.copy(); bad[0] = 1
    assert _create(a2a, 9, bad, col) == a2a.ERR_INVALID_ARG
    bad = rp.copy(); bad[4] = bad[3] - 1
    assert _create(a2a, 9, bad, col) == a2a.ERR_INVALID_ARG
    bad = col.copy(); bad[5] = 9
    assert _create(a2a, 9, rp, bad) == a2a.ERR_INVALID_ARG
    bad = col.copy(); bad[5] = -1
    assert _create(a2a, 9, rp, bad) == a2a.ERR_INVALID_ARG
    bad = col.copy(); bad[rp[2]] = 2
    assert _create(a2a, 9, rp, bad) == a2a.ERR_SELF_LOOP
    lib = a2a.load_library()
    assert lib.a2a_topo_create(9, rp.ctypes.data, col.ctypes.data, None) == a2a.ERR_INVALID_ARG
    # more hosts than the 32-bit offsets of a batch's arrays cover: refused before row_ptr is walked
    assert _create(a2a, 4 * 1024 * 1024 + 1, rp, col) == a2a.ERR_NOT_IMPLEMENTED
    # well-formed input: ok on a GPU machine, a HIP error (never a crash) without a device
    assert _create(a2a, 9, rp, col) in (a2a.OK, a2a.ERR_HIP)


def test_null_handles_are_rejected(a2a):
    lib = a2a.load_library()
    assert lib.a2a_topo_info(None, None, None, None, None) == a2a.ERR_INVALID_ARG
    assert lib.a2a_workspace_bytes(None, 4, 0) == 0
    assert lib.a2a_distances(None, 0, 1, None, None, None, None, None, None, 0, None) == a2a.ERR_INVALID_ARG
    assert lib.a2a_link_loads(None, 0, 1, None, None, None, None, 0, None) == a2a.ERR_INVALID_ARG
    out = a2a.Bound()
    assert lib.a2a_schedule_bound(None, None, 0, 0, 1.0, 1.0, ctypes.byref(out), None) == a2a.ERR_INVALID_ARG
    outc = a2a.BoundCap()
    assert lib.a2a_schedule_bound_cap(None, None, None, 0, 0, 1.0, 1.0, ctypes.byref(outc),
                                      None) == a2a.ERR_INVALID_ARG
    lib.a2a_topo_destroy(None)


def test_bound_struct_matches_header(a2a):
    text = open(os.path.join(ROOT, "include", "a2a_topo.h")).read()
    body = re.search(r"typedef struct a2a_bound \{(.*?)\} a2a_bound;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:double|int64_t|int32_t)\s+([a-z_]+);", body)
    assert fields == [n for n, _ in a2a.Bound._fields_]
    assert ctypes.sizeof(a2a.Bound) == 8 * 13
    body = re.search(r"typedef struct a2a_bound_cap \{(.*?)\} a2a_bound_cap;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"\b(?:double|int64_t|int32_t)\s+([a-z_]+);", body)
    assert fields == [n for n, _ in a2a.BoundCap._fields_]
    assert ctypes.sizeof(a2a.BoundCap) == 8 * 15
