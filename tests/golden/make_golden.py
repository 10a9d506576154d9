"""Writes tests/golden/fa_small_cases.json: results of the CPU oracle (oracle/fa_oracle.py,
nothing else) on small seeded inputs, as a regression record for the oracle itself and as
ready-made expected values for the library.

The paper prints no numeric value for any aggregator output (its results are accuracy curves),
so there is nothing to cite here; every number below is computed by the oracle, whose
arithmetic is pinned independently in tests/test_oracle_pins.py.

Run from the repository root:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth_inputs as si                      # noqa: E402
from oracle import fa_literal, fa_literal_grouped, as_f64_matrix   # noqa: E402

CASES = [
    # (name, p, n, m, lambda, iters, seed)
    ("tiny_p3", 3, 12, 2, 1.0, 6, 1),
    ("p7_lam0", 7, 40, 4, 0.0, 8, 2),
    ("p7_lam1", 7, 40, 4, 1.0, 8, 2),
    ("p16", 16, 64, 8, 1.0, 10, 3),
    ("p20", 20, 80, 9, 0.5, 10, 4),
    ("p33", 33, 120, 17, 1.0, 6, 5),
]

GROUPED_CASES = [
    # (name, block widths, n, m, lambda, iters, seed): workers that send several gradients
    ("grouped_mixed", [2, 3, 1, 2, 2], 60, 4, 1.0, 6, 6),
    ("grouped_equal", [3, 3, 3, 3], 50, 5, 1.0, 6, 7),
]


def build():
    rec = {}
    for name, p, n, m, lam, iters, seed in CASES:
        Gw = si.random_dense(p, n, seed=seed)
        res = fa_literal(as_f64_matrix(Gw), m, lam, iters, 0.0)
        rec[name] = {"p": p, "n": n, "m": m, "lambda": lam, "iters": iters, "seed": seed,
                     "out": [float(x) for x in res["out"]],
                     "v": [float(x) for x in res["v"]],
                     "objective": [float(x) for x in res["objective"]]}
    for name, sizes, n, m, lam, iters, seed in GROUPED_CASES:
        Gw = si.random_dense(sum(sizes), n, seed=seed)
        res = fa_literal_grouped(as_f64_matrix(Gw), sizes, m, lam, iters, 0.0)
        rec[name] = {"sizes": sizes, "p": sum(sizes), "n": n, "m": m, "lambda": lam,
                     "iters": iters, "seed": seed,
                     "out": [float(x) for x in res["out"]],
                     "v": [float(x) for x in res["v"]],
                     "objective": [float(x) for x in res["objective"]]}
    return rec


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "fa_small_cases.json")
    with open(path, "w") as f:
        json.dump(build(), f, indent=1)
    print("wrote", path)
