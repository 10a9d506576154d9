"""The seeded input generators: determinism, layout, and the stated recipes."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import decode_bf16


@pytest.mark.parametrize("name", list(si.WORKLOADS))
def test_shapes_determinism_and_byzantine_count(name):
    w = si.WORKLOADS[name].with_n(4096)
    a, ma = si.make_inputs(w, 0)
    b, mb = si.make_inputs(w, 0)
    c, _ = si.make_inputs(w, 1)
    assert a.shape == (w.p, 4096) and a.flags.c_contiguous
    assert a.dtype == (np.float32 if w.dtype == "f32" else np.uint16)
    assert np.array_equal(a, b) and ma == mb and not np.array_equal(a, c)
    assert len(ma["byzantine"]) == w.f == len(set(ma["byzantine"]))


def test_cfg1_recipe():
    w = si.WORKLOADS["cfg1"].with_n(20000)
    G, meta = si.make_inputs(w, 0)
    b = meta["byzantine"][0]
    honest = [i for i in range(w.p) if i != b]
    mu_est = G[honest].astype(np.float64).mean(axis=0)
    # Byzantine column is -10 mu; honest columns are mu + 0.1 noise
    assert np.abs(G[b] / -10.0 - mu_est).std() < 0.1
    resid = G[honest[0]].astype(np.float64) - mu_est
    assert 0.07 < resid.std() < 0.12


def test_cfg2_attack_kinds():
    w = si.WORKLOADS["cfg2"].with_n(20000)
    for seed in range(4):
        G, meta = si.make_inputs(w, seed)
        for b, kind in zip(meta["byzantine"], meta["byz_kinds"]):
            col = G[b].astype(np.float64)
            if kind == 2:
                assert abs(np.linalg.norm(col) - 1000.0) < 1e-2


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 37.0
    bits = si.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(decode_bf16(bits), ref)
