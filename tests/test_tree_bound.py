"""Theorem 1 (Sec. 5.4): the tree lower bound, on the CPU (host arithmetic of the library vs the
oracle's plain definition vs the paper's closed form)."""
import pytest

from helpers import paper_values


@pytest.fixture(scope="module")
def a2a():
    import os
    import paper_2309_13541_amd as lib
    if not os.path.exists(lib.library_path()):
        lib.build_library()
    lib.load_library()
    return lib


def closed_form(d, k):
    return eval(paper_values()["thm1_formula"], {"d": d, "k": k})


@pytest.mark.parametrize("d,k", [(2, 3), (2, 10), (3, 4), (4, 7), (8, 5), (16, 4)])
def test_full_trees_match_the_paper_formula(a2a, oracle, d, k):
    N = (d ** k - 1) // (d - 1)
    want = closed_form(d, k)
    assert want == sum(i * d ** i for i in range(k))
    assert oracle.tree_sum(N, d) == want
    tb = a2a.tree_lower_bound(N, d)
    assert tb.s_min == want and tb.full == 1 and tb.height == k - 1


@pytest.mark.parametrize("N,d", [(1, 4), (2, 1), (10, 1), (27, 6), (64, 4), (100, 3), (1000, 7),
                                 (16384, 4), (65536, 8), (99999, 2), (5462, 4)])
def test_partial_trees_match_the_definition(a2a, oracle, N, d):
    tb = a2a.tree_lower_bound(N, d, 2.0 ** 20, 3.125e9)
    assert tb.s_min == oracle.tree_sum(N, d)
    assert tb.t_lb == pytest.approx(tb.s_min * 2.0 ** 20 / (d * 3.125e9), rel=1e-15)
    if N > 1:
        assert tb.throughput_ub == pytest.approx((N - 1) * 2.0 ** 20 / tb.t_lb, rel=1e-15)
    else:
        assert tb.s_min == 0 and tb.height == 0


def test_known_values(a2a):
    assert a2a.tree_lower_bound(16384, 4).s_min == 107409   # levels 1,4,...,4^6 full, 10923 hosts at level 7
    assert a2a.tree_lower_bound(65536, 8).s_min == 350418
    assert a2a.tree_lower_bound(5461, 4).full == 1 and a2a.tree_lower_bound(5462, 4).full == 0


def test_bad_arguments(a2a):
    for args in [(0, 4, 1.0, 1.0), (5, 0, 1.0, 1.0), (5, 2, 0.0, 1.0), (5, 2, 1.0, -1.0)]:
        with pytest.raises(a2a.A2AError) as e:
            a2a.tree_lower_bound(*args)
        assert e.value.status == a2a.ERR_INVALID_ARG
