"""Writes oracle_config_values.json: summary figures and sampled link loads of the five
benchmark topologies, computed by the CPU oracle alone (never by the HIP path).

    python tests/golden/make_oracle_values.py [threads]

The full C5 run takes a few minutes on 8 cores.
"""
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import a2a_inputs as gen  # noqa: E402
import oracle  # noqa: E402

SAMPLES = 257  # link ids (k * E) // SAMPLES


def main():
    threads = int(sys.argv[1]) if len(sys.argv) > 1 else os.cpu_count()
    oracle.build(force=False)
    out = {"_written_by": "tests/golden/make_oracle_values.py (oracle/ only)"}
    for name in gen.CONFIG_NAMES:
        rp, col = gen.named_config(name)
        E = len(col)
        r = oracle.run(rp, col, threads=threads)
        ecc = oracle.run(rp, col, 0, 1, want_dist=True, want_load=False).dist.max()
        b = oracle.bound(rp, r.load, int(r.dist_sum.sum()))
        ids = [(k * E) // SAMPLES for k in range(SAMPLES)]
        out[name] = {
            "N": len(rp) - 1, "E": E,
            "sum_dist": int(r.dist_sum.sum()),
            "dist_sum_min": int(r.dist_sum.min()), "dist_sum_max": int(r.dist_sum.max()),
            "ecc_node0": int(ecc),
            "unreachable": int(r.unreachable), "flags": int(r.flags),
            "max_load": float(b["max_load"]).hex(), "argmax_arc": b["argmax_arc"],
            "min_load": float(b["min_load"]).hex(),
            "load_sum": float(r.load.sum()).hex(),
            "ratio_links": float(b["max_load"] * E / r.dist_sum.sum()),
            "sample_ids": ids,
            "sample_loads": [float(r.load[i]).hex() for i in ids],
        }
        print(name, {k: v for k, v in out[name].items() if not k.startswith("sample")}, flush=True)
    with open(os.path.join(HERE, "oracle_config_values.json"), "w") as f:
        json.dump(out, f, indent=1)


if __name__ == "__main__":
    main()
