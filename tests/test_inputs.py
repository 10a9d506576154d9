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


@pytest.mark.parametrize("name", ["cfg4", "cfg5"])
def test_chunked_generator_is_deterministic_and_follows_the_recipe(name):
    """The parallel generator of the two widest configurations: the same array whatever the
    thread count, ragged last chunk included, and the recipe's structure."""
    w = si.WORKLOADS[name].with_n(3 * 4096 + 77)
    a, ma = si.make_inputs_chunked(w, 0, threads=1, chunk_rows=4096)
    b, mb = si.make_inputs_chunked(w, 0, threads=5, chunk_rows=4096)
    c, _ = si.make_inputs_chunked(w, 1, threads=5, chunk_rows=4096)
    assert a.shape == (w.p, w.n) and a.flags.c_contiguous
    assert a.dtype == (np.float32 if w.dtype == "f32" else np.uint16)
    assert np.array_equal(a, b) and ma == mb and not np.array_equal(a, c)
    byz = ma["byzantine"]
    assert len(byz) == w.f == len(set(byz))
    G = (decode_bf16(a) if a.dtype == np.uint16 else a).astype(np.float64)
    honest = [i for i in range(w.p) if i not in byz]
    # honest columns are centre + noise of sigma = 0.5 rms(centre): their norms sit near
    # sqrt(1.25 n) (cfg5) or above it (cfg4 adds the low-rank part); large-norm noise columns
    # have sigma 5, i.e. norm near 5 sqrt(n)
    norms = np.linalg.norm(G, axis=1) / np.sqrt(w.n)
    assert np.all(norms[honest] > 1.0)
    big = [i for i in byz if norms[i] > 4.5]
    if name == "cfg4":
        assert len(big) == w.f and np.all(np.abs(norms[big] - 5.0) < 0.2)
        # rank: honest columns minus their mean live in span(U) + noise; 4 large singular values
        H = G[honest] - G[honest].mean(axis=0)
        sv = np.linalg.svd(H, compute_uv=False)
        assert sv[3] > 2.0 * sv[4]
    else:
        flips = [i for i in byz if i not in big]
        assert len(big) == w.f // 2 and len(flips) == w.f - w.f // 2
        assert np.array_equal(a[flips[0]], a[flips[1]])      # exact duplicates: -4 mu_1
        # two clusters: the honest columns correlate strongly within a cluster only
        C = np.corrcoef(G[honest])
        assert (C > 0.7).sum() > len(honest) and (C < 0.2).sum() > 0
