"""The stored oracle figures (tests/golden/oracle_config_values.json) are reproducible."""
import json
import os

import numpy as np
import pytest

import a2a_inputs as gen
from helpers import GOLDEN


@pytest.fixture(scope="module")
def stored():
    with open(os.path.join(GOLDEN, "oracle_config_values.json")) as f:
        return json.load(f)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4"])
def test_small_configs_reproduce(oracle, stored, name):
    rp, col = gen.named_config(name)
    r = oracle.run(rp, col, threads=8)
    g = stored[name]
    assert int(r.dist_sum.sum()) == g["sum_dist"]
    assert int(r.dist_sum.min()) == g["dist_sum_min"] and int(r.dist_sum.max()) == g["dist_sum_max"]
    got = r.load[np.asarray(g["sample_ids"])]
    want = np.array([float.fromhex(x) for x in g["sample_loads"]])
    np.testing.assert_allclose(got, want, rtol=1e-12)  # thread count changes summation order
    assert float(r.load.max()) == pytest.approx(float.fromhex(g["max_load"]), rel=1e-12)


def test_stored_values_are_consistent(stored):
    """Sum of loads = sum of distances; C4 loads are whole numbers (unique shortest paths)."""
    for name in gen.CONFIG_NAMES:
        g = stored[name]
        assert float.fromhex(g["load_sum"]) == pytest.approx(g["sum_dist"], rel=1e-12)
        assert g["unreachable"] == 0 and g["flags"] == 0
    c4 = stored["C4"]
    assert float.fromhex(c4["max_load"]) == 36402.0 and float.fromhex(c4["min_load"]) == 5461.0
    assert stored["C5"]["E"] == 524283
