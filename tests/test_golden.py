"""The stored small cases (tests/golden/fa_small_cases.json, written by
tests/golden/make_golden.py from the oracle alone): the oracle still reproduces them, and the
library matches them."""
import json
import os

import numpy as np
import pytest

import synth_inputs as si
from oracle import as_f64_matrix, fa_literal, fa_literal_grouped

HERE = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(HERE, "golden", "fa_small_cases.json")) as f:
    GOLDEN = json.load(f)


@pytest.mark.parametrize("name", sorted(GOLDEN))
def test_oracle_reproduces_the_stored_cases(name):
    g = GOLDEN[name]
    Gw = si.random_dense(g["p"], g["n"], seed=g["seed"])
    if "sizes" in g:
        res = fa_literal_grouped(as_f64_matrix(Gw), g["sizes"], g["m"], g["lambda"], g["iters"], 0.0)
    else:
        res = fa_literal(as_f64_matrix(Gw), g["m"], g["lambda"], g["iters"], 0.0)
    assert np.allclose(res["out"], g["out"], rtol=0, atol=1e-9 * np.abs(g["out"]).max())
    assert np.allclose(res["v"], g["v"], atol=1e-9)
    assert np.allclose(res["objective"], g["objective"], atol=1e-9)


@pytest.mark.gpu
@pytest.mark.parametrize("name", sorted(GOLDEN))
def test_library_matches_the_stored_cases(name):
    from gpu_util import announce, rel_l2, to_device
    from paper_2302_05865_amd import FlagAggregator
    announce("golden", name)
    g = GOLDEN[name]
    Gw = si.random_dense(g["p"], g["n"], seed=g["seed"])
    agg = FlagAggregator(n_max=g["n"], p_max=g["p"])
    if "sizes" in g:
        out = agg.fa_aggregate_grouped(to_device(Gw), g["sizes"], g["m"], g["lambda"], g["iters"],
                                       0.0).cpu().numpy()
    else:
        out = agg.fa_aggregate(to_device(Gw), g["m"], g["lambda"], g["iters"], 0.0).cpu().numpy()
    info = agg.fa_get_info()
    assert info.status == 0
    assert rel_l2(out.astype(np.float64), np.array(g["out"])) <= 1e-4
    v = info.v
    if "sizes" in g:                     # one value per worker: that of its first column
        v = v[np.concatenate([[0], np.cumsum(g["sizes"])[:-1]])]
    assert np.allclose(v, g["v"], atol=1e-6)
    assert np.allclose(info.objective, g["objective"], atol=1e-6)
    agg.close()
