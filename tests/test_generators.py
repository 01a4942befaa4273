import numpy as np
import pytest

import a2a_inputs as gen


def test_config_sizes():
    expect = {"C1": (64, 256), "C2": (1024, 10240), "C3": (4096, 24576), "C4": (16384, 65532)}
    for name, (N, E) in expect.items():
        rp, col = gen.named_config(name)
        assert rp.dtype == np.int32 and col.dtype == np.int32
        assert len(rp) - 1 == N and len(col) == E and rp[-1] == E


def test_torus_arc_order():
    rp, col = gen.torus([8, 8])
    assert list(col[rp[0]:rp[1]]) == [1, 7, 8, 56]
    assert list(col[rp[63]:rp[64]]) == [56, 62, 7, 55]


def test_hypercube_arc_order():
    rp, col = gen.hypercube(3)
    assert list(col[rp[5]:rp[6]]) == [4, 7, 1]


def test_imase_itoh_self_loops_dropped():
    rp, col = gen.imase_itoh(16384, 4)
    src = np.repeat(np.arange(16384), np.diff(rp))
    assert not np.any(src == col)
    assert np.sum(np.diff(rp) == 3) == 4
    # row 1: (-4-1, -4-2, -4-3, -4-4) mod N
    assert list(col[rp[1]:rp[2]]) == [16379, 16378, 16377, 16376]


def test_lcg_first_values():
    g = gen.lcg_stream(1234)
    x1 = (1234 * 6364136223846793005 + 1442695040888963407) % (1 << 64)
    x2 = (x1 * 6364136223846793005 + 1442695040888963407) % (1 << 64)
    assert next(g) == x1 >> 11 and next(g) == x2 >> 11


def test_random_regular_structure():
    N, d = 4096, 8
    rp, col = gen.random_regular(N, d, 99)
    src = np.repeat(np.arange(N), np.diff(rp))
    assert not np.any(src == col)
    # each permutation contributes in-degree exactly 1 => in-degree + dropped self loops = d
    indeg = np.bincount(col, minlength=N)
    outdeg = np.diff(rp)
    assert np.all(indeg == outdeg)  # node i loses one in- and one out-arc per fixed point


def test_c5_shape():
    rp, col = gen.named_config("C5")
    assert len(rp) - 1 == 65536
    assert len(col) == 65536 * 8 - int(np.sum(8 - np.diff(rp)))
    assert int(np.max(np.diff(rp))) == 8


def test_remove_arcs_and_nodes():
    t = gen.torus([3, 3])
    rp, col = gen.remove_arcs(t, [0, 35])
    assert rp[-1] == 34 and list(col[rp[0]:rp[1]]) == [2, 3, 6]
    rp2, col2 = gen.remove_nodes(t, [4])
    assert len(rp2) - 1 == 8 and rp2[-1] == 36 - 8
    assert col2.max() == 7


def test_torus_rejects_side_one():
    with pytest.raises(ValueError):
        gen.torus([1, 4])
