"""Parity of the HIP path against the fp64 CPU oracle, through the C ABI.

Gate (fp32 storage): relative L2 error of the aggregate <= 1e-4 and projector difference
||P_gpu - P_oracle||_F <= 1e-4 on Y, on the same seeded inputs.  The single kernels are held
to what their arithmetic allows: the Gram matrix accumulated in fp64 from exact products
<= 1e-12 relative to sqrt(K_ii K_jj); the Gram matrix from the bf16 matrix core (32-row sums
rounded to fp32 once, then fp64) a few fp32 roundings of a partial, see GRAM_LP_TOL; the
aggregate pass rounds an fp64 sum to fp32 once (<= 2^-23 relative per element).
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import (as_f64_matrix, basis_products, fa_literal, fa_literal_grouped, fa_scaled,
                    multi_krum, projector_difference)
from paper_2302_05865_amd import FaError, FlagAggregator

from gpu_util import announce, rel_l2, to_device

pytestmark = pytest.mark.gpu

GATE = 1e-4


# The default accumulation of the Gram pass switches to the bf16 matrix core at 2^20 rows; the
# cases here are smaller, so the contexts ask for that route by name ("bf16": wherever the
# kernel covers the case) or for fp64 accumulation.
@pytest.fixture(scope="module")
def agg_f32():
    a = FlagAggregator(n_max=1 << 22, p_max=64, dtype="f32", gram="bf16")
    yield a
    a.close()


@pytest.fixture(scope="module")
def agg_bf16():
    a = FlagAggregator(n_max=1 << 22, p_max=64, dtype="bf16", gram="bf16")
    yield a
    a.close()


@pytest.fixture(scope="module")
def agg_f32_fp64gram():
    a = FlagAggregator(n_max=1 << 22, p_max=64, dtype="f32", gram="fp64")
    yield a
    a.close()


@pytest.fixture(scope="module")
def agg_bf16_fp64gram():
    a = FlagAggregator(n_max=1 << 22, p_max=64, dtype="bf16", gram="fp64")
    yield a
    a.close()


def gram_tol(p, n, dtype, mode):
    """Bound on |K - G^T G| / sqrt(K_ii K_jj) by accumulation route.  fp64 accumulation of
    exact products: 1e-12.  bf16 matrix core (bf16 storage; fp32 storage at p > 16, when the
    context asks for it or, by default, from 2^20 rows on): each 32-row partial is rounded to fp32 once (six times for the
    pieces of fp32 values), |error| <= a few 2^-24 of the partial's sqrt(K_ii K_jj) share, and
    the shares add up to at most sqrt(K_ii K_jj): 2^-21 whatever n.  From a few thousand rows on
    the roundings average out and what is left is the measured bias of sums of squares,
    3.5e-9: held to 2e-8."""
    lp = mode == "bf16" and (dtype == "bf16" or p > 16)
    if not lp:
        return 1e-12
    return 2.0 ** -21 if n < 4096 else 2e-8


# ----------------------------------------------------------------------------- K1 + K2
# fp32 storage at p <= 16 accumulates in fp64 whatever the context asks for: one mode there
@pytest.mark.parametrize("p,mode", [(p, mode) for p in (1, 2, 7, 15, 16, 17, 31, 32, 33, 48, 64)
                                    for mode in ("bf16", "fp64") if p > 16 or mode == "bf16"])
@pytest.mark.parametrize("n", [1, 3, 255, 257, 4099, 300_001])
def test_gram_matches_fp64_definition(agg_f32, agg_f32_fp64gram, p, n, mode):
    announce("gram f32", mode, p, n)
    agg = agg_f32 if mode == "bf16" else agg_f32_fp64gram
    Gw = si.random_dense(p, n, seed=p * 1000 + n % 997, scale=3.0)
    K = agg.fa_gram(to_device(Gw))
    G = as_f64_matrix(Gw)
    ref = G.T @ G
    scale = np.sqrt(np.outer(np.diag(ref), np.diag(ref))) + 1e-300
    assert np.max(np.abs(K - ref) / scale) <= gram_tol(p, n, "f32", mode)
    assert np.array_equal(K, K.T)


@pytest.mark.parametrize("mode", ["bf16", "fp64"])
@pytest.mark.parametrize("p", [3, 16, 32, 40, 64])
@pytest.mark.parametrize("n", [5, 1023, 100_003])
def test_gram_bf16_storage(agg_bf16, agg_bf16_fp64gram, p, n, mode):
    announce("gram bf16", mode, p, n)
    agg = agg_bf16 if mode == "bf16" else agg_bf16_fp64gram
    Gw = si.f32_to_bf16_bits(si.random_dense(p, n, seed=p + n, scale=2.0).reshape(-1)).reshape(p, n)
    K = agg.fa_gram(to_device(Gw))
    G = as_f64_matrix(Gw)
    ref = G.T @ G
    scale = np.sqrt(np.outer(np.diag(ref), np.diag(ref))) + 1e-300
    assert np.max(np.abs(K - ref) / scale) <= gram_tol(p, n, "bf16", mode)
    assert np.array_equal(K, K.T)


@pytest.mark.parametrize("dtype,p", [("f32", 40), ("bf16", 12)])
def test_default_gram_route_switches_at_the_documented_size(agg_f32, agg_bf16, agg_f32_fp64gram,
                                                            agg_bf16_fp64gram, dtype, p):
    """fa_config.gram = FA_GRAM_AUTO: fp64 accumulation below FA_GRAM_AUTO_MIN_ROWS rows, the
    bf16 matrix core from there on -- bit for bit what the contexts that name the route return."""
    from paper_2302_05865_amd._ctypes_defs import FA_GRAM_AUTO_MIN_ROWS
    auto = FlagAggregator(n_max=FA_GRAM_AUTO_MIN_ROWS + 8, p_max=p, dtype=dtype)
    named_fp64 = agg_f32_fp64gram if dtype == "f32" else agg_bf16_fp64gram
    named_bf16 = agg_f32 if dtype == "f32" else agg_bf16
    for n, named in ((FA_GRAM_AUTO_MIN_ROWS - 1, named_fp64), (FA_GRAM_AUTO_MIN_ROWS, named_bf16)):
        announce("default gram route", dtype, p, n)
        Gw = si.random_dense(p, n, seed=n % 1000 + p, scale=1.3)
        if dtype == "bf16":
            Gw = si.f32_to_bf16_bits(Gw.reshape(-1)).reshape(p, n)
        dev = to_device(Gw)
        assert np.array_equal(auto.fa_gram(dev), named.fa_gram(dev))
    # and the two routes differ at all at this size (else the comparison shows nothing)
    assert not np.array_equal(named_fp64.fa_gram(dev), named_bf16.fa_gram(dev))
    auto.close()


@pytest.mark.parametrize("dtype,p,n", [("bf16", 15, 70_001), ("bf16", 64, 50_003),
                                       ("f32", 40, 60_001), ("f32", 64, 33_333)])
def test_matrix_core_gram_keeps_duplicates_exact_and_is_reproducible(agg_f32, agg_bf16, dtype,
                                                                      p, n):
    """The bf16 matrix-core Gram pass: identical gradients -- in one 16-column block or in
    different ones -- must give bitwise identical entries K_ii = K_ij = K_jj (the pair is then
    recognised as a duplicate, D_ij = 0 exactly), and two runs the same bits.  With bf16
    storage the whole rows of two duplicates agree bit for bit; with fp32 storage the products
    of the pieces are added in an order that depends on which of the two columns comes first,
    so there the rows agree to the pass's accuracy only."""
    announce("gram lp duplicates", dtype, p, n)
    Gw = si.random_dense(p, n, seed=77 + p, scale=1.7)
    pairs = [(0, 1), (2, p - 1), (p // 2, p // 2 + 1)]
    for i, j in pairs:
        Gw[j] = Gw[i]
    agg = agg_f32
    if dtype == "bf16":
        Gw = si.f32_to_bf16_bits(Gw.reshape(-1)).reshape(p, n)
        agg = agg_bf16
    dev = to_device(Gw)
    K1 = agg.fa_gram(dev)
    K2 = agg.fa_gram(dev)
    assert np.array_equal(K1, K2)
    for i, j in pairs:
        assert K1[i, i] == K1[i, j] == K1[j, j] == K1[j, i]
        if dtype == "bf16":
            assert np.array_equal(K1[i], K1[j])
        else:
            scale = np.sqrt(K1[i, i] * np.diag(K1))
            assert np.max(np.abs(K1[i] - K1[j]) / scale) <= 2e-8


def test_gram_with_row_stride_and_determinism(agg_f32):
    announce("gram strided")
    p, n, ld = 15, 70_001, 70_016
    Gw = si.random_dense(p, ld, seed=5)
    dev = torch.from_numpy(Gw).cuda()[:, :n]
    assert dev.stride(0) == ld
    K1 = agg_f32.fa_gram(dev)
    K2 = agg_f32.fa_gram(dev)
    G = as_f64_matrix(Gw[:, :n])
    ref = G.T @ G
    assert np.max(np.abs(K1 - ref)) <= 1e-12 * np.abs(ref).max()
    assert np.array_equal(K1, K2)          # fixed-order reduction: bitwise reproducible


# -------------------------------------------- Gram matrix built as the gradients arrive
@pytest.mark.parametrize("name,n", [("cfg1", 33_333), ("cfg2", 100_003), ("cfg4", 60_001),
                                    ("cfg5", 20_011)])
def test_gram_built_on_arrival_equals_the_one_shot_path(name, n):
    """fa_gram_begin / fa_gram_update / fa_aggregate_arrived: the gradients land one by one in
    a buffer whose other places still hold NaN (they must not be read); each arrival extends K
    by one row and column.  At the end K is the fp64 Gram matrix (<= 1e-12) and the aggregate
    is the oracle's, and fa_aggregate's on the assembled buffer."""
    announce("gram on arrival", name, n)
    w = si.WORKLOADS[name].with_n(n)
    Gw, _ = si.make_inputs(w, 3)
    full = to_device(Gw)
    nan = np.full(Gw.shape, 0x7FC0, np.uint16) if Gw.dtype == np.uint16 else \
        np.full(Gw.shape, np.nan, np.float32)
    buf = to_device(nan)                      # same 16-byte row pitch as `full`
    assert torch.isnan(buf.float()).all()
    agg = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype, gram="fp64")
    agg.fa_gram_begin(w.p, w.n)
    order = np.random.default_rng(5).permutation(w.p)
    for i in order:
        buf[i] = full[i]
        agg.fa_gram_update(buf, int(i))
    with pytest.raises(FaError):
        agg.fa_gram_update(buf, int(order[0]))            # announced twice
    out = agg.fa_aggregate_arrived(buf, w.m, w.lam, w.iters, 0.0)
    info = agg.fa_get_info()
    G = as_f64_matrix(Gw)
    Kref = G.T @ G
    scale = np.sqrt(np.outer(np.diag(Kref), np.diag(Kref)))
    assert info.status == 0
    assert np.max(np.abs(info.K - Kref) / scale) <= 1e-12
    ref = fa_scaled(Gw, w.m, w.lam, w.iters, 0.0)
    got = out.cpu().numpy().astype(np.float64)
    assert rel_l2(got, ref["out"]) <= GATE
    assert projector_difference(info.A, ref["A"], ref["R"]) <= GATE
    one_shot = agg.fa_aggregate(full, w.m, w.lam, w.iters, 0.0).cpu().numpy().astype(np.float64)
    assert rel_l2(got, one_shot) <= 1e-6
    with pytest.raises(FaError):                            # the round is over
        agg.fa_aggregate_arrived(buf, w.m, w.lam, w.iters, 0.0)
    agg.close()


@pytest.mark.parametrize("name,n,pieces", [("cfg2", 100_003, 5), ("cfg4", 60_001, 3),
                                          ("cfg5", 20_011, 4), ("cfg1", 33_333, 16)])
def test_gram_built_from_pieces_of_gradients(name, n, pieces):
    """fa_gram_update_rows: every gradient lands in `pieces` pieces (same cuts for all, each on a
    16-byte boundary), the pieces of different gradients interleaved at random; places that have
    not landed hold NaN.  K ends up the fp64 Gram matrix and the aggregate the oracle's."""
    announce("gram from pieces", name, n, pieces)
    w = si.WORKLOADS[name].with_n(n)
    Gw, _ = si.make_inputs(w, 4)
    full = to_device(Gw)
    nan = np.full(Gw.shape, 0x7FC0, np.uint16) if Gw.dtype == np.uint16 else \
        np.full(Gw.shape, np.nan, np.float32)
    buf = to_device(nan)
    cuts = [0] + [int(round(n * k / pieces / 8)) * 8 for k in range(1, pieces)] + [n]
    agg = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype, gram="fp64")
    agg.fa_gram_begin(w.p, w.n)
    rng = np.random.default_rng(9)
    nxt = np.zeros(w.p, dtype=int)              # next piece of each gradient
    events = []
    while (nxt < pieces).any():
        i = int(rng.choice(np.flatnonzero(nxt < pieces)))
        events.append((i, int(nxt[i])))
        nxt[i] += 1
    for i, c in events:
        r0, r1 = cuts[c], cuts[c + 1]
        buf[i, r0:r1] = full[i, r0:r1]
        agg.fa_gram_update_rows(buf, i, r0, r1 - r0)
    out = agg.fa_aggregate_arrived(buf, w.m, w.lam, w.iters, 0.0)
    info = agg.fa_get_info()
    G = as_f64_matrix(Gw)
    Kref = G.T @ G
    scale = np.sqrt(np.outer(np.diag(Kref), np.diag(Kref)))
    assert info.status == 0
    assert np.max(np.abs(info.K - Kref) / scale) <= 1e-12
    assert np.array_equal(info.K, info.K.T)
    ref = fa_scaled(Gw, w.m, w.lam, w.iters, 0.0)
    assert rel_l2(out.cpu().numpy().astype(np.float64), ref["out"]) <= GATE
    assert projector_difference(info.A, ref["A"], ref["R"]) <= GATE
    agg.close()


def test_gram_from_pieces_argument_errors():
    announce("gram from pieces: errors")
    dev = to_device(si.random_dense(3, 1000, seed=8))
    agg_f32 = FlagAggregator(n_max=1000, p_max=3)
    agg_f32.fa_gram_begin(3, 1000)
    with pytest.raises(FaError):
        agg_f32.fa_gram_update_rows(dev, 0, 8, 100)          # does not start where the last piece ended
    agg_f32.fa_gram_update_rows(dev, 0, 0, 400)
    with pytest.raises(FaError):
        agg_f32.fa_gram_update_rows(dev, 0, 0, 400)          # the same piece twice
    with pytest.raises(FaError):
        agg_f32.fa_gram_update_rows(dev, 1, 0, 600)          # gradient 0 ends inside this piece
    with pytest.raises(FaError):
        agg_f32.fa_gram_update_rows(dev, 0, 400, 601)        # past the end
    agg_f32.fa_gram_update_rows(dev, 1, 0, 400)
    agg_f32.fa_gram_update_rows(dev, 1, 400, 101)            # may end anywhere ...
    with pytest.raises(FaError):
        agg_f32.fa_gram_update_rows(dev, 1, 501, 100)        # ... but the next piece starts off a 16-byte boundary
    with pytest.raises(FaError):
        agg_f32.fa_aggregate_arrived(dev, 1, 0.0, 1, 0.0)    # nothing is complete yet
    agg_f32.fa_gram_begin(3, 1000)                           # a new round forgets the old one
    for i in range(3):
        agg_f32.fa_gram_update(dev, i)
    a = agg_f32.fa_aggregate_arrived(dev, 1, 0.0, 2, 0.0)
    b = agg_f32.fa_aggregate(dev, 1, 0.0, 2, 0.0)
    assert rel_l2(a.cpu().numpy().astype(np.float64), b.cpu().numpy().astype(np.float64)) <= 1e-6
    agg_f32.close()


def test_gram_on_arrival_argument_errors(agg_f32):
    announce("gram on arrival: errors")
    dev = to_device(si.random_dense(5, 1000, seed=8))
    with pytest.raises(FaError):
        agg_f32.fa_gram_update(dev, 0)                      # no round open
    agg_f32.fa_gram_begin(5, 1000)
    with pytest.raises(FaError):
        agg_f32.fa_gram_update(dev, 5)                      # no such gradient
    for i in range(4):
        agg_f32.fa_gram_update(dev, i)
    with pytest.raises(FaError):                            # gradient 4 is still missing
        agg_f32.fa_aggregate_arrived(dev, 2, 1.0, 3, 0.0)
    agg_f32.fa_gram_update(dev, 4)
    a = agg_f32.fa_aggregate_arrived(dev, 2, 1.0, 3, 0.0)
    b = agg_f32.fa_aggregate(dev, 2, 1.0, 3, 0.0)
    assert rel_l2(a.cpu().numpy().astype(np.float64), b.cpu().numpy().astype(np.float64)) <= 1e-6
    with pytest.raises(FaError):
        agg_f32.fa_gram_begin(65, 1000)


# ---------------------------------------------------------------------------------- K4
@pytest.mark.parametrize("p", [1, 7, 15, 16, 33, 64])
@pytest.mark.parametrize("n", [1, 6, 1025, 250_003])
def test_combine_matches_definition(agg_f32, p, n):
    announce("combine f32", p, n)
    Gw = si.random_dense(p, n, seed=p + 17 * (n % 101))
    c = np.random.default_rng(p).standard_normal(p)
    out = agg_f32.fa_combine(to_device(Gw), c).cpu().numpy()
    ref = as_f64_matrix(Gw) @ c
    tol = 2.0 ** -23 * np.abs(as_f64_matrix(Gw)) @ np.abs(c) + 1e-30
    assert np.all(np.abs(out - ref) <= tol)


@pytest.mark.parametrize("p,n", [(5, 9), (32, 100_001)])
def test_combine_bf16_storage(agg_bf16, p, n):
    announce("combine bf16", p, n)
    Gw = si.f32_to_bf16_bits(si.random_dense(p, n, seed=3).reshape(-1)).reshape(p, n)
    c = np.random.default_rng(p).standard_normal(p)
    out = agg_bf16.fa_combine(to_device(Gw), c).cpu().numpy()
    ref = as_f64_matrix(Gw) @ c
    # bf16 storage accumulates in fp32 with c rounded to fp32: p + 1 roundings, each at most
    # 2^-24 of the sum of the terms' magnitudes
    tol = (p + 2) * 2.0 ** -24 * np.abs(as_f64_matrix(Gw)) @ np.abs(c) + 1e-30
    assert np.all(np.abs(out - ref) <= tol)


# ---------------------------------------------------------------------------------- K3
@pytest.mark.parametrize("name,n", [("cfg1", 20000), ("cfg2", 50000), ("cfg3", 50000),
                                    ("cfg4", 30000), ("cfg5", 20000)])
def test_irls_kernel_from_oracle_gram(agg_f32, name, n):
    """The p x p kernel alone, fed the oracle's Gram matrix: isolates K3 from K1's rounding."""
    announce("irls", name, n)
    w = si.WORKLOADS[name].with_n(n)
    Gw, _ = si.make_inputs(w, 0)
    ref = fa_scaled(Gw, w.m, w.lam, w.iters, 0.0)
    agg_f32.fa_irls(ref["K"], w.m, w.lam, w.iters, 0.0)
    info = agg_f32.fa_get_info()
    assert info.status == 0 and info.iters_done == w.iters
    G = as_f64_matrix(Gw)
    assert rel_l2(G @ info.c, ref["out"]) <= 1e-9
    assert projector_difference(info.A, ref["A"], ref["R"]) <= 1e-9
    assert np.allclose(info.objective, ref["objective"], atol=1e-6)
    assert np.allclose(info.v, ref["v"], atol=1e-9)


# ------------------------------------------------------------------------- end to end
def _check_aggregate(agg, w, seed, lam=None, n_gate=GATE):
    lam = w.lam if lam is None else lam
    Gw, meta = si.make_inputs(w, seed)
    ref = fa_scaled(Gw, w.m, lam, w.iters, 0.0)
    dev = to_device(Gw)
    out = agg.fa_aggregate(dev, w.m, lam, w.iters, 0.0)
    info = agg.fa_get_info()
    got = out.cpu().numpy().astype(np.float64)
    e_out = rel_l2(got, ref["out"])
    e_proj = projector_difference(info.A, ref["A"], ref["R"])
    announce(w.name, "seed", seed, "lam", lam, "rel_l2", e_out, "proj", e_proj, "gap",
             info.eigengap, "rank", info.rank, "sweeps", info.sweeps)
    assert info.status == 0 and info.iters_done == w.iters
    assert e_out <= n_gate
    assert e_proj <= n_gate
    assert np.allclose(info.v, ref["v"], atol=1e-6)
    return info


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("lam", [0.0, 1.0])
def test_aggregate_cfg1_full_size(agg_f32, seed, lam):
    _check_aggregate(agg_f32, si.WORKLOADS["cfg1"], seed, lam)


@pytest.mark.parametrize("seed", [0, 1])
@pytest.mark.parametrize("name,n", [("cfg2", 700_003), ("cfg3", 500_001)])
def test_aggregate_p15_reduced_n(agg_f32, name, n, seed):
    _check_aggregate(agg_f32, si.WORKLOADS[name].with_n(n), seed)


@pytest.mark.parametrize("lam", [0.0, 0.1, 1.0])
def test_aggregate_cfg5_reduced_n(agg_f32, lam):
    _check_aggregate(agg_f32, si.WORKLOADS["cfg5"].with_n(300_007), 0, lam)


def test_aggregate_cfg4_bf16_reduced_n(agg_bf16):
    _check_aggregate(agg_bf16, si.WORKLOADS["cfg4"].with_n(400_003), 0)


# ---------------------------------------------------------------------- special cases
def test_full_subspace_returns_the_mean(agg_f32):
    announce("m = p -> mean")
    Gw = si.random_dense(9, 50_001, seed=11)
    out = agg_f32.fa_aggregate(to_device(Gw), 9, 1.0, 5, 0.0).cpu().numpy()
    assert rel_l2(out, as_f64_matrix(Gw).mean(axis=1)) <= 1e-6


def test_identical_gradients_return_the_gradient(agg_f32):
    announce("identical gradients")
    g = si.random_dense(1, 40_003, seed=12)
    Gw = np.repeat(g, 6, axis=0)
    out = agg_f32.fa_aggregate(to_device(Gw), 3, 1.0, 4, 0.0).cpu().numpy()
    info = agg_f32.fa_get_info()
    assert info.rank == 1
    assert rel_l2(out, g[0].astype(np.float64)) <= 1e-6


def test_single_worker_and_tiny_n(agg_f32):
    announce("p = 1, tiny n")
    for n in (1, 2, 5):
        Gw = si.random_dense(1, n, seed=n)
        out = agg_f32.fa_aggregate(to_device(Gw), 1, 1.0, 3, 0.0).cpu().numpy()
        assert rel_l2(out, Gw[0].astype(np.float64)) <= 1e-6
    Gw = si.random_dense(4, 3, seed=9)          # n < p: rank 3
    ref = fa_literal(as_f64_matrix(Gw), 2, 1.0, 4, 0.0)
    out = agg_f32.fa_aggregate(to_device(Gw), 2, 1.0, 4, 0.0).cpu().numpy()
    assert rel_l2(out, ref["out"]) <= GATE


def test_zero_column_and_duplicate_columns(agg_f32):
    announce("zero column + duplicates")
    Gw = si.random_dense(7, 30_001, seed=13)
    Gw[2] = 0.0
    Gw[5] = Gw[1]
    ref = fa_scaled(Gw, 3, 1.0, 6, 0.0)
    out = agg_f32.fa_aggregate(to_device(Gw), 3, 1.0, 6, 0.0).cpu().numpy()
    info = agg_f32.fa_get_info()
    assert info.rank == 5 and info.w[2] == 0.0
    assert rel_l2(out, ref["out"]) <= GATE


def test_nonfinite_and_all_zero_inputs(agg_f32):
    announce("nan / zero input")
    Gw = si.random_dense(5, 10_000, seed=14)
    Gw[3, 777] = np.nan
    out = agg_f32.fa_aggregate(to_device(Gw), 2, 1.0, 3, 0.0).cpu().numpy()
    assert agg_f32.fa_get_info().status == 4 and np.all(np.isnan(out))
    Gw = np.zeros((5, 10_000), dtype=np.float32)
    out = agg_f32.fa_aggregate(to_device(Gw), 2, 1.0, 3, 0.0).cpu().numpy()
    assert agg_f32.fa_get_info().status == 5 and np.all(out == 0)


def test_tol_stops_like_the_oracle(agg_f32):
    announce("tol stop")
    w = si.WORKLOADS["cfg1"].with_n(50_000)
    Gw, _ = si.make_inputs(w, 3)
    ref = fa_scaled(Gw, w.m, 1.0, 50, 1e-4)
    out = agg_f32.fa_aggregate(to_device(Gw), w.m, 1.0, 50, 1e-4).cpu().numpy()
    info = agg_f32.fa_get_info()
    assert info.iters_done == ref["iters_done"] < 50
    assert rel_l2(out, ref["out"]) <= GATE


def test_bitwise_reproducible(agg_f32):
    announce("determinism")
    w = si.WORKLOADS["cfg2"].with_n(400_001)
    Gw, _ = si.make_inputs(w, 4)
    dev = to_device(Gw)
    a = agg_f32.fa_aggregate(dev, w.m, w.lam, w.iters, 0.0).clone()
    b = agg_f32.fa_aggregate(dev, w.m, w.lam, w.iters, 0.0)
    assert torch.equal(a, b)


def test_basis_is_orthonormal_and_matches_oracle_subspace(agg_f32):
    announce("fa_basis")
    w = si.WORKLOADS["cfg2"].with_n(200_001)
    Gw, _ = si.make_inputs(w, 0)
    dev = to_device(Gw)
    agg_f32.fa_aggregate(dev, w.m, w.lam, w.iters, 0.0)
    Y = agg_f32.fa_basis(dev, w.m).cpu().numpy().astype(np.float64).T      # n x m
    assert np.abs(Y.T @ Y - np.eye(w.m)).max() <= 1e-5
    ref = fa_scaled(Gw, w.m, w.lam, w.iters, 0.0)
    Yo = as_f64_matrix(Gw) @ ref["A"]
    cos = np.linalg.svd(Yo.T @ Y, compute_uv=False)
    assert np.all(np.abs(cos - 1) <= 1e-5)
    # a buffer sized for another m than the last solve's is refused, nothing is written
    for wrong_m in (w.m - 1, w.m + 1):
        with pytest.raises(FaError):
            agg_f32.fa_basis(dev, wrong_m)


def test_argument_errors(agg_f32):
    announce("argument errors")
    dev = to_device(si.random_dense(4, 100, seed=1))
    with pytest.raises(FaError):
        agg_f32.fa_aggregate(dev, 0, 1.0, 3, 0.0)
    with pytest.raises(FaError):
        agg_f32.fa_aggregate(dev, 5, 1.0, 3, 0.0)
    with pytest.raises(FaError):
        agg_f32.fa_aggregate(dev, 2, -1.0, 3, 0.0)
    with pytest.raises(FaError):
        agg_f32.fa_aggregate(dev, 2, 1.0, 0, 0.0)
    with pytest.raises(FaError):
        agg_f32.fa_aggregate(dev, 2, 1.0, 3, -1.0)
    with pytest.raises(FaError):
        agg_f32.fa_aggregate(dev[:, 1:], 2, 1.0, 3, 0.0)       # misaligned base pointer
    with pytest.raises(FaError):
        agg_f32.fa_aggregate(torch.zeros((4, 99), device="cuda"), 2, 1.0, 3, 0.0)  # row pitch
    small = FlagAggregator(n_max=50, p_max=4)
    with pytest.raises(FaError):
        small.fa_aggregate(dev, 2, 1.0, 3, 0.0)                 # n > n_max
    small.close()
    with pytest.raises(TypeError):
        agg_f32.fa_aggregate(dev.double(), 2, 1.0, 3, 0.0)


# ------------------------------------------------------------- solver paths of the p x p part
@pytest.mark.parametrize("solver", ["jacobi16", "jacobi"])
def test_alternative_pxp_solvers_agree_with_the_oracle(solver):
    """p <= 16 has three p x p solvers (purification by default, the wave-level Jacobi
    path, the generic Jacobi kernel); fa_config.solver picks one."""
    announce("solver", solver)
    agg = FlagAggregator(n_max=1 << 20, p_max=16, dtype="f32", solver=solver)
    _check_aggregate(agg, si.WORKLOADS["cfg2"].with_n(300_007), 5)
    _check_aggregate(agg, si.WORKLOADS["cfg1"].with_n(40_001), 5)
    agg.close()


def test_tied_eigenvalues_fall_back_and_give_a_valid_subspace(agg_f32):
    """Orthogonal gradients of equal norm: every eigenvalue of the weighted PCA ties, the
    minimiser is not unique and purification cannot separate the spectrum.  What is unique
    is checked (Y orthonormal, sum of explained variances = m, out = G c)."""
    announce("tied eigenvalues")
    p, n, m = 6, 6 * 1000, 3
    Gw = np.zeros((p, n), dtype=np.float32)
    for i in range(p):
        Gw[i, i * 1000:(i + 1) * 1000] = 1.0
    out = agg_f32.fa_aggregate(to_device(Gw), m, 1.0, 5, 0.0).cpu().numpy().astype(np.float64)
    info = agg_f32.fa_get_info()
    assert info.status == 0 and info.rank == p
    K = as_f64_matrix(Gw).T @ as_f64_matrix(Gw)
    assert np.abs(info.A.T @ K @ info.A - np.eye(m)).max() <= 1e-10
    assert abs(info.v.sum() - m) <= 1e-9 and info.v.min() >= -1e-12 and info.v.max() <= 1 + 1e-12
    assert rel_l2(out, as_f64_matrix(Gw) @ info.c) <= 1e-6
    P = info.A @ info.A.T @ K                      # coefficients of Y Y^T G
    assert np.allclose(info.c, P.sum(axis=1) / p, atol=1e-10)


def test_single_kernels_enqueued_one_by_one_equal_the_whole_call(agg_f32):
    announce("fa_gram_async / fa_enqueue_kernel")
    w = si.WORKLOADS["cfg2"].with_n(123_457)
    Gw, _ = si.make_inputs(w, 6)
    dev = to_device(Gw)
    whole = agg_f32.fa_aggregate(dev, w.m, w.lam, w.iters, 0.0).clone()
    K_whole = agg_f32.fa_get_info().K.copy()
    agg_f32.fa_gram_async(dev)
    out = torch.zeros_like(whole)
    agg_f32.fa_enqueue_kernel(2, dev, w.m, w.lam, w.iters, 0.0, out=out)
    agg_f32.fa_enqueue_kernel(3, dev, w.m, w.lam, w.iters, 0.0, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out, whole)
    assert np.array_equal(agg_f32.fa_gram(dev), K_whole)


# ---------------------------------------------------------------- re-streaming schedule
def _check_restream(agg, w, seed, n_gate=GATE):
    Gw, _ = si.make_inputs(w, seed)
    ref = fa_scaled(Gw, w.m, w.lam, w.iters, 0.0)
    dev = to_device(Gw)
    once = agg.fa_aggregate(dev, w.m, w.lam, w.iters, 0.0).clone()
    out = agg.fa_aggregate_restream(dev, w.m, w.lam, w.iters)
    info = agg.fa_get_info()
    _, v_s, obj_s = agg.fa_get_restream_info()
    got = out.cpu().numpy().astype(np.float64)
    e_once = rel_l2(got, once.cpu().numpy().astype(np.float64))
    e_out = rel_l2(got, ref["out"])
    e_proj = projector_difference(info.A, ref["A"], ref["R"])
    announce("restream", w.name, "vs gram-once", e_once, "vs oracle", e_out, "proj", e_proj,
             "max |v_streamed - v|", np.abs(v_s - ref["v"]).max())
    assert info.status == 0 and info.iters_done == w.iters
    assert e_once <= 1e-5 and e_out <= n_gate and e_proj <= n_gate
    # the streamed explained variances and the streamed objective are the oracle's
    assert np.allclose(v_s, ref["v"], atol=1e-6)
    assert np.allclose(obj_s[:w.iters], ref["objective"], atol=1e-5)
    assert np.allclose(info.objective, ref["objective"], atol=1e-5)


@pytest.mark.parametrize("name,n", [("cfg1", 100_000), ("cfg2", 300_007), ("cfg3", 200_001)])
def test_restream_schedule_matches_gram_once_and_oracle(agg_f32, name, n):
    """Two passes over G per IRLS solve (weighted Gram, streamed projections) must give what
    the two-pass default schedule gives."""
    _check_restream(agg_f32, si.WORKLOADS[name].with_n(n), 0)


def test_restream_schedule_largest_p(agg_f32):
    _check_restream(agg_f32, si.WORKLOADS["cfg5"].with_n(60_001).with_lam(1.0), 0)


def test_restream_schedule_bf16(agg_bf16):
    _check_restream(agg_bf16, si.WORKLOADS["cfg4"].with_n(80_003), 0)


def test_restream_with_duplicate_and_zero_columns(agg_f32):
    announce("restream: zero column + duplicates")
    Gw = si.random_dense(7, 30_001, seed=13)
    Gw[2] = 0.0
    Gw[5] = Gw[1]
    ref = fa_scaled(Gw, 3, 1.0, 6, 0.0)
    out = agg_f32.fa_aggregate_restream(to_device(Gw), 3, 1.0, 6).cpu().numpy()
    assert agg_f32.fa_get_info().rank == 5
    assert rel_l2(out, ref["out"]) <= GATE


# ------------------------------------------------- the 16 < p <= 64 matrix-core p x p solver
@pytest.mark.parametrize("mode", ["fp64", "bf16"])
@pytest.mark.parametrize("p,m", [(17, 9), (24, 5), (33, 17), (40, 20), (48, 47), (64, 32)])
@pytest.mark.parametrize("lam", [0.0, 1.0])
def test_wide_problems_all_tile_counts(agg_f32, agg_f32_fp64gram, p, m, lam, mode):
    """Orders 32, 48 and 64 of the tiled solver (2 x 2, 3 x 3, 4 x 4 tiles), ragged p.  With the
    Gram matrix accumulated in fp64 the p x p solver is held to 1e-6; with the default route of
    these widths (bf16 matrix core, K good to ~1e-8 at this small n, which the subspace
    amplifies by up to 1e3) the whole path is held to the gate."""
    announce("wide", mode, p, m, lam)
    tol = 1e-6 if mode == "fp64" else GATE
    agg_f32 = agg_f32 if mode == "bf16" else agg_f32_fp64gram
    rng = np.random.default_rng(p)
    n = 20_011
    mu = rng.standard_normal(n)
    Gw = (mu[None, :] + 0.7 * rng.standard_normal((p, n))).astype(np.float32)
    Gw[1] = -3.0 * mu                      # a Byzantine column
    Gw[p - 1] = Gw[2]                      # a duplicate: rank p - 1
    ref = fa_scaled(Gw, m, lam, 8, 0.0)
    out = agg_f32.fa_aggregate(to_device(Gw), m, lam, 8, 0.0).cpu().numpy().astype(np.float64)
    info = agg_f32.fa_get_info()
    assert info.status == 0 and info.rank == p - 1 and info.iters_done == 8
    assert rel_l2(out, ref["out"]) <= tol
    assert projector_difference(info.A, ref["A"], ref["R"]) <= tol
    # (with m = rank every residual is exactly zero here; the oracle's SVD leaves square
    # roots of rounding noise, ~1e-6 in total)
    assert np.allclose(info.objective, ref["objective"], atol=5 * tol)
    assert np.allclose(info.v, ref["v"], atol=tol)


def test_wide_problem_with_tied_eigenvalues_uses_the_standby_solver(agg_f32):
    """p = 20 orthogonal gradients of equal norm: the purification cannot converge, the
    Jacobi kernel takes over; what is unique is checked."""
    announce("wide, tied eigenvalues")
    p, m = 20, 7
    Gw = np.zeros((p, p * 500), dtype=np.float32)
    for i in range(p):
        Gw[i, i * 500:(i + 1) * 500] = 1.0
    out = agg_f32.fa_aggregate(to_device(Gw), m, 1.0, 4, 0.0).cpu().numpy().astype(np.float64)
    info = agg_f32.fa_get_info()
    G = as_f64_matrix(Gw)
    K = G.T @ G
    assert info.status == 0 and info.rank == p
    assert np.abs(info.A.T @ K @ info.A - np.eye(m)).max() <= 1e-10
    assert abs(info.v.sum() - m) <= 1e-9
    assert rel_l2(out, G @ info.c) <= 1e-6


def test_wide_problem_on_the_jacobi_kernel():
    announce("wide, Jacobi kernel")
    agg = FlagAggregator(n_max=1 << 20, p_max=64, dtype="f32", solver="jacobi")
    _check_aggregate(agg, si.WORKLOADS["cfg5"].with_n(30_001).with_lam(1.0), 3)
    agg.close()


@pytest.mark.parametrize("name,n", [("cfg4", 60_001), ("cfg5", 30_001)])
def test_wide_solver_gives_up_and_the_jacobi_kernel_redoes_the_solve(name, n):
    """A spin budget of zero makes the first wait for a steering word of the matrix-core solver
    (16 < p <= 64) give up; every wavefront then leaves the purification at the same barrier,
    the kernel hands over, and the Jacobi kernel enqueued behind it must return the oracle's
    answer.  Every kernel exits normally."""
    announce("wide solver gives up", name)
    w = si.WORKLOADS[name].with_n(n)
    agg = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype, wide_spin_budget=0)
    info = _check_aggregate(agg, w, 1)
    ref = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype, solver="jacobi")
    info_j = _check_aggregate(ref, w, 1)
    # Jacobi sweeps, not purification steps: the stand-by did the work, with the very
    # arithmetic of a context that asks for the Jacobi kernel outright
    assert info.sweeps == info_j.sweeps
    assert np.array_equal(info.c, info_j.c)
    agg.close()
    ref.close()


def test_wide_problem_nonfinite_and_tol(agg_f32):
    announce("wide: nan, tol")
    Gw = si.random_dense(33, 5_000, seed=21)
    ref = fa_scaled(Gw, 12, 1.0, 40, 1e-5)
    out = agg_f32.fa_aggregate(to_device(Gw), 12, 1.0, 40, 1e-5).cpu().numpy()
    info = agg_f32.fa_get_info()
    assert info.iters_done == ref["iters_done"] < 40 and rel_l2(out, ref["out"]) <= GATE
    assert np.isfinite(info.eigengap) and info.eigengap > 0
    Gw[5, 17] = np.inf
    out = agg_f32.fa_aggregate(to_device(Gw), 12, 1.0, 3, 0.0).cpu().numpy()
    assert agg_f32.fa_get_info().status == 4 and np.all(np.isnan(out))


# ------------------------------------------------------------ general exponent (Sec. 2.2)
@pytest.mark.parametrize("a", [1.0, 1.5, 4.0])
@pytest.mark.parametrize("name,n", [("cfg2", 100_003), ("cfg5", 20_001)])
def test_general_exponent(name, n, a):
    """Terms (1 - v)^(1/a) with the Taylor constant a of Sec. 2.2 other than FA's a = 2."""
    announce("exponent", a, name)
    w = si.WORKLOADS[name].with_n(n).with_lam(1.0)
    Gw, _ = si.make_inputs(w, 2)
    iters = 10
    ref = fa_scaled(Gw, w.m, w.lam, iters, 0.0, a=a)
    agg = FlagAggregator(n_max=w.n, p_max=w.p, exponent_a=a)
    dev = to_device(Gw)
    out = agg.fa_aggregate(dev, w.m, w.lam, iters, 0.0).cpu().numpy().astype(np.float64)
    info = agg.fa_get_info()
    assert info.status == 0
    assert rel_l2(out, ref["out"]) <= GATE
    assert projector_difference(info.A, ref["A"], ref["R"]) <= GATE
    assert np.allclose(info.objective, ref["objective"], atol=1e-6)
    if name == "cfg2":
        out2 = agg.fa_aggregate_restream(dev, w.m, w.lam, iters).cpu().numpy().astype(np.float64)
        assert rel_l2(out2, ref["out"]) <= GATE
    # every solver knows the exponent: the purification solvers (p <= 16 and wide), the Jacobi
    # eigensolver of the p <= 16 kernel and the any-p kernel -- all routes, one answer
    for solver in (("jacobi16", "jacobi") if w.p <= 16 else ("jacobi",)):
        other = FlagAggregator(n_max=w.n, p_max=w.p, exponent_a=a, solver=solver)
        out3 = other.fa_aggregate(dev, w.m, w.lam, iters, 0.0).cpu().numpy().astype(np.float64)
        assert other.fa_get_info().status == 0
        assert rel_l2(out3, out) <= 1e-6, solver
        assert np.allclose(other.fa_get_info().objective, info.objective, atol=1e-9), solver
        other.close()
    agg.close()


# --------------------------------------------------- interleaved (row-major) storage of G
def _rows_device(Gw, pitch=None):
    """[p, n] host array -> device tensor [n, pitch][:, :p] (coordinate k's values contiguous)."""
    p, n = Gw.shape
    pitch = pitch or p
    if Gw.dtype == np.uint16:
        t = torch.zeros((n, pitch), dtype=torch.bfloat16, device="cuda")
        t[:, :p] = torch.from_numpy(np.ascontiguousarray(Gw.T).view(np.int16)).cuda().view(torch.bfloat16)
    else:
        t = torch.zeros((n, pitch), dtype=torch.float32, device="cuda")
        t[:, :p] = torch.from_numpy(np.ascontiguousarray(Gw.T)).cuda()
    return t[:, :p]


@pytest.mark.parametrize("p,pitch", [(1, 1), (3, 3), (7, 8), (15, 15), (15, 16), (16, 16), (17, 17),
                                      (31, 32), (40, 44), (64, 64)])
@pytest.mark.parametrize("n", [1, 5, 255, 1031, 70_001])
def test_row_major_gram_and_combine(p, pitch, n):
    announce("row-major gram/combine", p, pitch, n)
    agg = FlagAggregator(n_max=1 << 20, p_max=64, layout="row_major")
    Gw = si.random_dense(p, n, seed=100 + p)
    dev = _rows_device(Gw, pitch)
    G = as_f64_matrix(Gw)
    K = agg.fa_gram(dev)
    ref = G.T @ G
    scale = np.sqrt(np.outer(np.diag(ref), np.diag(ref)))
    assert np.abs(K - ref).max() <= 1e-12 * scale.max()
    c = np.random.default_rng(p).standard_normal(p)
    out = agg.fa_combine(dev, c).cpu().numpy().astype(np.float64)
    want = G @ c
    assert np.abs(out - want).max() <= 2.0 ** -23 * np.abs(G).max() * np.abs(c).sum() + 1e-30
    agg.close()


@pytest.mark.parametrize("name,n", [("cfg1", 100_000), ("cfg2", 300_007), ("cfg5", 30_001)])
def test_row_major_aggregate(name, n):
    announce("row-major aggregate", name)
    w = si.WORKLOADS[name].with_n(n).with_lam(1.0)
    Gw, _ = si.make_inputs(w, 0)
    ref = fa_scaled(Gw, w.m, w.lam, w.iters, 0.0)
    agg = FlagAggregator(n_max=w.n, p_max=w.p, layout="row_major")
    dev = _rows_device(Gw)
    out = agg.fa_aggregate(dev, w.m, w.lam, w.iters, 0.0).cpu().numpy().astype(np.float64)
    info = agg.fa_get_info()
    assert info.status == 0
    assert rel_l2(out, ref["out"]) <= GATE
    assert projector_difference(info.A, ref["A"], ref["R"]) <= GATE
    Y = agg.fa_basis(dev, w.m).cpu().numpy().astype(np.float64).T
    assert np.abs(Y.T @ Y - np.eye(w.m)).max() <= 1e-5
    with pytest.raises(FaError):
        agg.fa_aggregate_restream(dev, w.m, w.lam, 2)
    agg.close()


def test_row_major_bf16():
    announce("row-major bf16")
    w = si.WORKLOADS["cfg4"].with_n(50_003)
    Gw, _ = si.make_inputs(w, 0)
    ref = fa_scaled(Gw, w.m, w.lam, w.iters, 0.0)
    agg = FlagAggregator(n_max=w.n, p_max=w.p, dtype="bf16", layout="row_major")
    out = agg.fa_aggregate(_rows_device(Gw), w.m, w.lam, w.iters, 0.0).cpu().numpy()
    assert rel_l2(out, ref["out"]) <= GATE
    agg.close()


# ---- streamed check of a materialised basis (Y^T Y, Y^T G on the device) -----------------------
@pytest.mark.parametrize("name,n,layout", [
    ("cfg1", 100_000, "worker_major"), ("cfg2", 262_147, "worker_major"),
    ("cfg2", 4_099, "row_major"), ("cfg3", 65_537, "worker_major"),
    ("cfg4", 70_001, "worker_major"), ("cfg4", 20_011, "row_major"),
    ("cfg5", 40_003, "worker_major"), ("cfg2", 13, "worker_major"), ("cfg2", 1, "worker_major")])
def test_check_basis_matches_the_definition(name, n, layout):
    announce("fa_check_basis", name, n, layout)
    w = si.WORKLOADS[name].with_n(n)
    Gw, _ = si.make_inputs(w, 0)
    agg = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype, layout=layout)
    dev = _rows_device(Gw) if layout == "row_major" else to_device(Gw)
    agg.fa_aggregate(dev, w.m, w.lam, min(w.iters, 4), 0.0)
    Y = agg.fa_basis(dev, w.m)
    YtY, YtG = agg.fa_check_basis(dev, Y)
    # the definition, on exactly the numbers the device holds (Y is stored in fp32)
    G64 = as_f64_matrix(Gw)
    Y64 = Y.cpu().numpy().astype(np.float64).T
    rYY, rYG = basis_products(G64, Y64)
    scale_g = np.sqrt((G64 ** 2).sum(axis=0)).max()
    assert np.abs(YtY - rYY).max() <= 1e-11
    assert np.abs(YtG - rYG).max() <= 1e-11 * max(scale_g, 1.0)
    # and what it is for: the basis is orthonormal (to the fp32 storage of Y), and the
    # explained variances of the last solve come back from Y^T G
    if n > w.p:
        assert np.abs(YtY - np.eye(w.m)).max() <= 1e-5
        info = agg.fa_get_info()
        s = (G64 ** 2).sum(axis=0)
        assert np.allclose((YtG ** 2).sum(axis=0) / s, info.v, atol=1e-5)
    agg.close()


def test_check_basis_of_any_matrix_and_argument_errors(agg_f32):
    announce("fa_check_basis free Y")
    rng = np.random.default_rng(5)
    n, p, m = 5_003, 15, 3
    Gw = si.random_dense(p, n, seed=7)
    dev = to_device(Gw)
    Yh = rng.standard_normal((m, n)).astype(np.float32)
    Yd = torch.from_numpy(np.ascontiguousarray(np.pad(Yh, ((0, 0), (0, 1))))).cuda()[:, :n]
    YtY, YtG = agg_f32.fa_check_basis(dev, Yd)
    rYY, rYG = basis_products(as_f64_matrix(Gw), Yh.astype(np.float64).T)
    assert np.abs(YtY - rYY).max() <= 1e-9 and np.abs(YtG - rYG).max() <= 1e-9
    with pytest.raises(TypeError):
        agg_f32.fa_check_basis(dev, Yd[:, :-1])
    with pytest.raises(FaError):
        agg_f32.fa_check_basis(dev, torch.zeros((p + 1, n), dtype=torch.float32, device="cuda"))
    with pytest.raises(FaError):                 # columns of Y off the 16-byte grid
        agg_f32.fa_check_basis(dev, torch.zeros((m, n + 2), dtype=torch.float32, device="cuda")[:, :n])


@pytest.mark.parametrize("p,m,dtype,layout", [
    (33, 5, "f32", "worker_major"), (20, 20, "bf16", "worker_major"), (40, 17, "f32", "row_major"),
    (64, 40, "f32", "worker_major"), (64, 64, "bf16", "worker_major"), (17, 1, "f32", "worker_major"),
    (64, 64, "f32", "row_major"), (48, 33, "bf16", "row_major")])
def test_check_basis_every_tile_shape(p, m, dtype, layout):
    """Any n x m matrix as Y: every count of 16-column tiles of Y and of G, both storage types and
    orders, a ragged number of rows; against the definition."""
    announce("fa_check_basis tiles", p, m, dtype, layout)
    rng = np.random.default_rng(p * 100 + m)
    n = 9_007
    Gw = si.random_dense(p, n, seed=p + m)
    if dtype == "bf16":
        Gw = (Gw.view(np.uint32) >> 16).astype(np.uint16)
    agg = FlagAggregator(n_max=n, p_max=p, dtype=dtype, layout=layout)
    dev = _rows_device(Gw) if layout == "row_major" else to_device(Gw)
    Yh = rng.standard_normal((m, n)).astype(np.float32)
    Yd = torch.from_numpy(np.ascontiguousarray(np.pad(Yh, ((0, 0), (0, 1))))).cuda()[:, :n]
    YtY, YtG = agg.fa_check_basis(dev, Yd)
    rYY, rYG = basis_products(as_f64_matrix(Gw), Yh.astype(np.float64).T)
    assert np.abs(YtY - rYY).max() <= 1e-9 and np.abs(YtG - rYG).max() <= 1e-9
    agg.close()


# ---- workers that send several gradients (blocks of columns) -----------------------------------
@pytest.mark.parametrize("sizes,m,lam,n,dtype", [
    ([2, 3, 1, 2, 2, 1, 4], 8, 1.0, 30_011, "f32"), ([4] * 8, 9, 1.0, 20_000, "f32"),
    ([1] * 15, 8, 1.0, 25_003, "f32"), ([3, 2, 3, 2, 3], 4, 0.0, 12_345, "f32"),
    ([8, 8, 8, 8, 8, 8, 8, 4], 20, 0.5, 9_001, "f32"), ([5, 5, 6], 3, 1.0, 16_384, "bf16"),
    ([7], 2, 1.0, 1_000, "f32"), ([16] * 4, 33, 1.0, 5_003, "f32"),
    ([3] * 5 + [1], 8, 2.0, 7_001, "f32")])
@pytest.mark.parametrize("solver", ["auto", "jacobi"])
def test_grouped_workers_match_the_block_oracle(sizes, m, lam, n, dtype, solver):
    """Both routes of the block solver: the matrix-core purification kernel (default) and the
    any-p Jacobi kernel."""
    announce("grouped", sizes, m, lam, n, dtype, solver)
    q = sum(sizes)
    Gw = si.random_dense(q, n, seed=q + m)
    Gw[0] += 1.5 * Gw[q - 1]
    if dtype == "bf16":
        Gw = (Gw.view(np.uint32) >> 16).astype(np.uint16)      # truncated to bf16 bits
    iters = 6
    ref = fa_literal_grouped(as_f64_matrix(Gw), sizes, m, lam, iters, 0.0)
    agg = FlagAggregator(n_max=n, p_max=q, dtype=dtype, solver=solver)
    out = agg.fa_aggregate_grouped(to_device(Gw), sizes, m, lam, iters, 0.0).cpu().numpy()
    info = agg.fa_get_info()
    assert info.status == 0 and info.iters_done == iters
    assert rel_l2(out.astype(np.float64), ref["out"]) <= GATE
    first = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    assert np.allclose(info.v[first], ref["v"], atol=1e-6)
    assert np.allclose(info.objective, ref["objective"], atol=1e-6)
    # every column reports its worker's value and weight
    owner = np.repeat(np.arange(len(sizes)), sizes)
    assert np.array_equal(info.v, info.v[first][owner])
    assert np.array_equal(info.w, info.w[first][owner])
    agg.close()


@pytest.mark.parametrize("a", [1.5, 4.0])
def test_grouped_workers_general_exponent(a):
    """Blocks of columns with the constant a of Sec. 2.2 Step 2 other than 2, both routes."""
    announce("grouped, exponent", a)
    sizes, m, lam, n, iters = [2, 2, 3, 3, 2, 1, 5], 7, 1.0, 9_973, 5
    q = sum(sizes)
    Gw = si.random_dense(q, n, seed=77)
    ref = fa_literal_grouped(as_f64_matrix(Gw), sizes, m, lam, iters, 0.0, a=a)
    outs = []
    for solver in ("auto", "jacobi"):
        agg = FlagAggregator(n_max=n, p_max=q, exponent_a=a, solver=solver)
        out = agg.fa_aggregate_grouped(to_device(Gw), sizes, m, lam, iters, 0.0).cpu().numpy()
        info = agg.fa_get_info()
        assert info.status == 0 and info.iters_done == iters
        assert rel_l2(out.astype(np.float64), ref["out"]) <= GATE
        assert np.allclose(info.objective, ref["objective"], atol=1e-6)
        outs.append(out)
        agg.close()
    assert rel_l2(outs[0].astype(np.float64), outs[1].astype(np.float64)) <= 1e-6


@pytest.mark.parametrize("name,n", [("cfg2", 100_003), ("cfg4", 50_021)])
def test_grouped_with_single_columns_is_fa_aggregate(name, n):
    announce("grouped = plain at k = 1", name)
    w = si.WORKLOADS[name].with_n(n)
    Gw, _ = si.make_inputs(w, 2)
    dev = to_device(Gw)
    # on the any-p solver the two entries run the same code: bit for bit
    gen = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype, solver="jacobi")
    a = gen.fa_aggregate_grouped(dev, [1] * w.p, w.m, w.lam, 5, 0.0).clone()
    b = gen.fa_aggregate(dev, w.m, w.lam, 5, 0.0).clone()
    assert torch.equal(a, b)
    gen.close()
    # on the default route the block kernel takes powers where the plain one has square roots
    plain = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype)
    c = plain.fa_aggregate_grouped(dev, [1] * w.p, w.m, w.lam, 5, 0.0).clone()
    info_c = plain.fa_get_info()
    d = plain.fa_aggregate(dev, w.m, w.lam, 5, 0.0)
    info_d = plain.fa_get_info()
    assert info_c.status == 0 and info_d.status == 0
    assert rel_l2(c.cpu().numpy().astype(np.float64), d.cpu().numpy().astype(np.float64)) <= 1e-6
    assert rel_l2(c.cpu().numpy().astype(np.float64), b.cpu().numpy().astype(np.float64)) <= 1e-6
    assert np.allclose(info_c.objective, info_d.objective, rtol=0, atol=1e-9)
    assert np.allclose(info_c.v, info_d.v, rtol=0, atol=1e-8)
    plain.close()


@pytest.mark.parametrize("sizes,m", [([4] * 10, 17), ([3, 3, 2, 2, 3], 6)])
def test_grouped_stand_by_redoes_the_solve_when_the_purification_gives_up(sizes, m):
    """The block solver's hand-over: with a spin budget of zero the purification kernel gives up
    at its first wait and the Jacobi kernel behind it answers, bit for bit what a context asking
    for that kernel returns.  Also on the block route: a worker sent twice (its pair is dropped,
    its columns are linearly dependent), non-finite and all-zero input."""
    q, n, iters = sum(sizes), 8_009, 4
    announce("grouped stand-by", sizes, m)
    Gw = si.random_dense(q, n, seed=31)
    dev = to_device(Gw)
    agg = FlagAggregator(n_max=n, p_max=q, wide_spin_budget=0)
    a = agg.fa_aggregate_grouped(dev, sizes, m, 1.0, iters, 0.0).clone()
    info = agg.fa_get_info()
    ref = FlagAggregator(n_max=n, p_max=q, solver="jacobi")
    b = ref.fa_aggregate_grouped(dev, sizes, m, 1.0, iters, 0.0)
    info_j = ref.fa_get_info()
    assert info.status == 0 and info_j.status == 0
    assert info.sweeps == info_j.sweeps and torch.equal(a, b)
    agg.close()
    ref.close()
    agg = FlagAggregator(n_max=n, p_max=q)
    twice = Gw.copy()
    twice[sizes[0]:2 * sizes[0]] = twice[0:sizes[0]]          # worker 1 = worker 0
    oracle = fa_literal_grouped(as_f64_matrix(twice), sizes, m, 1.0, iters, 0.0)
    out = agg.fa_aggregate_grouped(to_device(twice), sizes, m, 1.0, iters, 0.0).cpu().numpy()
    info = agg.fa_get_info()
    assert info.status == 0 and info.rank == q - sizes[0]
    assert rel_l2(out.astype(np.float64), oracle["out"]) <= GATE
    assert np.allclose(info.objective, oracle["objective"], atol=1e-6)
    bad = Gw.copy()
    bad[1, 5] = np.nan
    out = agg.fa_aggregate_grouped(to_device(bad), sizes, m, 1.0, iters, 0.0).cpu().numpy()
    assert agg.fa_get_info().status == 4 and np.all(np.isnan(out))
    out = agg.fa_aggregate_grouped(to_device(np.zeros_like(Gw)), sizes, m, 1.0, iters, 0.0).cpu().numpy()
    assert agg.fa_get_info().status == 5 and np.all(out == 0.0)
    agg.close()


def test_grouped_argument_errors(agg_f32):
    announce("grouped argument errors")
    dev = to_device(si.random_dense(6, 100, seed=1))
    for sizes in ([2, 2, 1], [2, 2, 3], [6, 0], [], [2, -1, 5]):
        with pytest.raises(FaError):
            agg_f32.fa_aggregate_grouped(dev, sizes, 2, 1.0, 3, 0.0)
    with pytest.raises(FaError):
        agg_f32.fa_aggregate_grouped(dev, [3, 3], 7, 1.0, 3, 0.0)


# ---- seeded sweep over shapes: every p x p path, many (p, m, lambda) ----------------------------
@pytest.mark.parametrize("seed", range(36))
def test_random_shapes_all_solvers(agg_f32, seed):
    rng = np.random.default_rng(1000 + seed)
    p = int(rng.integers(2, 65))
    m = int(rng.integers(1, p + 1))
    lam = float(rng.choice([0.0, 0.3, 1.0, 4.0]))
    iters = int(rng.integers(1, 9))
    n = int(rng.integers(p + 1, 6000))
    announce("random shape", seed, p, m, lam, iters, n)
    mu = rng.standard_normal(n)
    Gw = (mu[None, :] * rng.uniform(0.2, 2.0, p)[:, None] +
          rng.uniform(0.1, 1.5) * rng.standard_normal((p, n))).astype(np.float32)
    nbyz = int(rng.integers(0, max(1, p // 4) + 1))
    for b in rng.choice(p, size=nbyz, replace=False):
        Gw[b] = (-4.0 * mu if rng.random() < 0.5 else 30.0 * rng.standard_normal(n)).astype(np.float32)
    ref = fa_scaled(Gw, m, lam, iters, 0.0)
    out = agg_f32.fa_aggregate(to_device(Gw), m, lam, iters, 0.0).cpu().numpy().astype(np.float64)
    info = agg_f32.fa_get_info()
    assert info.status == 0 and info.iters_done == iters
    assert rel_l2(out, ref["out"]) <= GATE
    assert projector_difference(info.A, ref["A"], ref["R"]) <= GATE
    assert np.allclose(info.objective, ref["objective"], atol=2e-5)


# ---- Multi-Krum from the same Gram pass -----------------------------------------------------------
@pytest.mark.parametrize("name,n,f,q,layout", [
    ("cfg1", 50_000, 1, 6, "worker_major"), ("cfg2", 100_003, 3, 12, "worker_major"),
    ("cfg2", 100_003, 3, 1, "worker_major"), ("cfg2", 4_099, 3, 12, "row_major"),
    ("cfg3", 65_537, 3, 12, "worker_major"), ("cfg4", 30_001, 6, 26, "worker_major"),
    ("cfg5", 20_011, 12, 52, "worker_major"), ("cfg5", 20_011, 0, 64, "worker_major")])
def test_multi_krum_matches_the_published_rule(name, n, f, q, layout):
    announce("multi-krum", name, n, f, q, layout)
    w = si.WORKLOADS[name].with_n(n)
    Gw, _ = si.make_inputs(w, 0)
    ref = multi_krum(as_f64_matrix(Gw), f, q)
    agg = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype, layout=layout, gram="bf16")
    dev = _rows_device(Gw) if layout == "row_major" else to_device(Gw)
    out, scores, selected = agg.fa_multikrum(dev, f, q)
    # integer decisions: the same set (the workloads have no near-ties apart from exact
    # duplicates, which tie exactly on both sides and go to the smaller index)
    assert np.array_equal(selected, ref["selected"])
    # distances come from the Gram matrix: fp64 accumulation 1e-10; the bf16 matrix-core pass
    # of bf16 storage and of p > 16 (K good to a few 1e-9 of the norms) 1e-7
    stol = 1e-7 if (w.dtype == "bf16" or w.p > 16) and layout == "worker_major" else 1e-10
    assert np.allclose(scores, ref["scores"], rtol=stol, atol=stol * ref["scores"].max())
    assert rel_l2(out.cpu().numpy().astype(np.float64), ref["out"]) <= 1e-6
    agg.close()


def test_multi_krum_argument_errors_and_no_basis(agg_f32):
    announce("multi-krum argument errors")
    dev = to_device(si.random_dense(6, 100, seed=1))
    for f, q in ((4, 2), (-1, 2), (1, 0), (1, 7)):
        with pytest.raises(FaError):
            agg_f32.fa_multikrum(dev, f, q)
    agg_f32.fa_multikrum(dev, 1, 5)
    with pytest.raises(FaError):
        agg_f32.fa_basis(dev, 2)              # no basis belongs to a Multi-Krum result


@pytest.mark.parametrize("name,n", [("cfg2", 2_000_003), ("cfg5", 200_001)])
def test_two_contexts_on_two_streams_give_the_results_of_the_sequence(name, n):
    """Independent gradient sets, one context and one stream each, in flight together (the
    streaming passes of one beside the p x p solver of the other): every result is bit for bit
    what the same call returns when nothing else runs."""
    w = si.WORKLOADS[name].with_n(n)
    devs = [to_device(si.make_inputs(w, seed)[0]) for seed in (0, 1)]
    aggs = [FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype) for _ in range(2)]
    try:
        refs = []
        for i in range(2):
            refs.append(aggs[0].fa_aggregate(devs[i], w.m, w.lam, w.iters, 0.0).clone())
        torch.cuda.synchronize()
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        outs = [torch.empty_like(refs[0]) for _ in range(2)]
        announce(f"two streams {name} n={n}")
        for rep in range(6):
            for o in outs:
                o.fill_(float("nan"))
            torch.cuda.synchronize()
            for i in range(4):
                with torch.cuda.stream(streams[i & 1]):
                    aggs[i & 1].fa_aggregate(devs[i & 1], w.m, w.lam, w.iters, 0.0, out=outs[i & 1])
            torch.cuda.synchronize()
            for i in range(2):
                assert torch.equal(outs[i], refs[i]), (rep, i)
                assert aggs[i].fa_get_info().status == 0
    finally:
        for a in aggs:
            a.close()


# ---- degenerate shapes -----------------------------------------------------------------------------
@pytest.mark.parametrize("p,n,m", [(15, 5, 8), (15, 5, 3), (7, 1, 4), (7, 2, 1), (40, 9, 20),
                                   (40, 9, 4), (64, 3, 32), (2, 1, 1), (1, 10, 1), (1, 1, 1),
                                   (16, 16, 8), (17, 16, 9), (33, 31, 32)])
def test_fewer_coordinates_than_workers(p, n, m):
    """n < p (the rank is n), n = p, a single worker, a single coordinate: against the oracle,
    with and without the pairwise term."""
    announce("tiny shape", p, n, m)
    rng = np.random.default_rng(1000 * p + n)
    for lam in (0.0, 1.0):
        G = rng.standard_normal((p, n)).astype(np.float32)
        ref = fa_scaled(G, m, lam, 6, 0.0)
        agg = FlagAggregator(n_max=n, p_max=p)
        out = agg.fa_aggregate(to_device(G), m, lam, 6, 0.0).cpu().numpy().astype(np.float64)
        info = agg.fa_get_info()
        agg.close()
        assert info.status == 0 and info.rank == min(p, n)
        assert rel_l2(out, ref["out"]) <= GATE
        # (where Y spans all of G the terms are square roots of rounding noise: 1e-8 each)
        assert np.allclose(info.objective[:6], ref["objective"][:6], atol=1e-5)


@pytest.mark.parametrize("p,n,m", [(15, 20_011, 8), (32, 9_001, 16), (64, 5_003, 32)])
def test_extreme_scales_and_parameters(p, n, m):
    """Workers whose norms spread over twelve orders of magnitude or sit at 1e18 / 1e-18, a huge
    and a vanishing lambda, the largest solve count, m = 1 and m = p, identical gradients:
    against the oracle."""
    announce("extremes", p, n, m)
    rng = np.random.default_rng(11 + p)
    mu = rng.standard_normal(n)
    base = mu[None, :] + 0.5 * rng.standard_normal((p, n))
    same = base.copy()
    same[1:] = same[0]
    cases = [("spread", base * (10.0 ** rng.uniform(-6, 6, p))[:, None], m, 1.0, 10),
             ("1e18", base * 1e18, m, 1.0, 10), ("1e-18", base * 1e-18, m, 1.0, 10),
             ("lambda 1e6", base, m, 1e6, 10), ("lambda 1e-9", base, m, 1e-9, 10),
             ("64 solves", base, m, 1.0, 64), ("m = p", base, p, 1.0, 5), ("m = 1", base, 1, 1.0, 12),
             ("identical", same, m, 1.0, 5)]
    agg = FlagAggregator(n_max=n, p_max=p)
    for tag, G64, mm, lam, iters in cases:
        G = G64.astype(np.float32)
        ref = fa_scaled(G, mm, lam, iters, 0.0)
        out = agg.fa_aggregate(to_device(G), mm, lam, iters, 0.0).cpu().numpy().astype(np.float64)
        info = agg.fa_get_info()
        assert info.status == 0, tag
        assert rel_l2(out, ref["out"]) <= GATE, tag
        assert projector_difference(info.A, ref["A"], ref["R"]) <= GATE, tag
    agg.close()


@pytest.mark.parametrize("p,n,dtype,gram", [(32, 9_001, "f32", "bf16"), (64, 4_003, "f32", "bf16"),
                                            (15, 20_011, "bf16", "bf16"), (32, 9_001, "bf16", "bf16"),
                                            (32, (1 << 20) + 5, "bf16", "auto")])
def test_values_beyond_the_matrix_core_range_take_the_fp64_pass(p, n, dtype, gram):
    """A worker may send anything: values of 1e25 (finite in fp32 and in bf16) overflow the fp32
    sums of the bf16 matrix-core Gram pass; the fp64 pass standing by behind it redoes K, and
    the aggregate is the oracle's.  The same context then takes an ordinary input on the
    matrix-core route again."""
    announce("beyond the matrix-core range", p, n, dtype, gram)
    rng = np.random.default_rng(5 * p)
    mu = rng.standard_normal(n)
    G = (mu[None, :] + 0.5 * rng.standard_normal((p, n))).astype(np.float32)
    big = G.copy()
    big[3] = (1e25 * rng.standard_normal(n)).astype(np.float32)
    big[p - 1] *= np.float32(3e20)
    m, lam, iters = (p + 1) // 2, 1.0, 6
    agg = FlagAggregator(n_max=n, p_max=p, dtype=dtype, gram=gram)
    fp64 = FlagAggregator(n_max=n, p_max=p, dtype=dtype, gram="fp64")
    for Gf in (big, G, big):
        Gw = si.f32_to_bf16_bits(Gf.reshape(-1)).reshape(p, n) if dtype == "bf16" else Gf
        dev = to_device(Gw)
        ref = fa_scaled(Gw, m, lam, iters, 0.0)
        out = agg.fa_aggregate(dev, m, lam, iters, 0.0).cpu().numpy().astype(np.float64)
        info = agg.fa_get_info()
        assert info.status == 0
        assert rel_l2(out, ref["out"]) <= GATE
        if Gf is big:
            assert np.allclose(info.v, ref["v"], atol=1e-5)
            # the stand-by's K is the fp64 route's, bit for bit
            out64 = fp64.fa_aggregate(dev, m, lam, iters, 0.0)
            assert np.array_equal(info.K, fp64.fa_get_info().K)
            assert np.array_equal(out, out64.cpu().numpy().astype(np.float64))
    agg.close()
    fp64.close()


# ---- the enqueue-only entry points inside a HIP graph ------------------------------------------
@pytest.mark.parametrize("name,n,entry", [("cfg2", 300_007, "aggregate"),
                                          ("cfg4", 200_003, "aggregate"),
                                          ("cfg5", 60_013, "aggregate"),
                                          ("cfg2", 100_003, "restream"),
                                          ("cfg4", 100_003, "static")])
def test_enqueue_only_entry_points_recorded_into_a_graph(name, n, entry):
    """fa_aggregate, fa_aggregate_restream and fa_aggregate_static only launch kernels (what
    they clear, a fill kernel clears), so a caller may record them into a HIP graph.  The graph
    is replayed four times on changing inputs, with eager calls on the same workspace and
    synchronisations between the replays; every replay is bit for bit the eager result."""
    from paper_2302_05865_amd import fa_aggregate_static
    w = si.WORKLOADS[name].with_n(n)
    hosts = [si.make_inputs(w, seed)[0] for seed in (0, 1)]
    devs = [to_device(h) for h in hosts]
    Gin = to_device(hosts[0])                        # the graph's input buffer
    iters = min(w.iters, 4) if entry == "restream" else w.iters
    agg = FlagAggregator(n_max=w.n, p_max=w.p, dtype=w.dtype)

    def run(G, out):
        if entry == "aggregate":
            agg.fa_aggregate(G, w.m, w.lam, iters, 0.0, out=out)
        elif entry == "restream":
            agg.fa_aggregate_restream(G, w.m, w.lam, iters, out=out)
        else:
            fa_aggregate_static(G, w.m, w.lam, iters, 0.0, out)

    try:
        refs = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(2)]
        for i in range(2):
            run(devs[i], refs[i])
        torch.cuda.synchronize()
        assert agg.fa_get_info().status == 0 or entry == "static"
        out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        other = torch.empty_like(out)
        announce(f"graph capture {entry} {name} n={n}")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run(Gin, out)
        torch.cuda.synchronize()
        for rep in range(4):
            k = rep & 1
            out.fill_(float("nan"))
            other.fill_(float("nan"))
            Gin.copy_(devs[k])
            announce(f"graph replay {rep}")
            graph.replay()
            run(devs[1 - k], other)                  # eager work on the same workspace
            torch.cuda.synchronize()
            assert torch.equal(out, refs[k]), rep
            assert torch.equal(other, refs[1 - k]), rep
        del graph
    finally:
        agg.close()


# ---- random problems through every entry point and option -----------------------------------------
_ENTRY_KINDS = ["bf16", "row_major", "row_major_bf16", "exponent", "restream", "static", "arrival",
                "krum", "grouped", "stop_rule"]


@pytest.mark.parametrize("seed", range(60))
def test_random_problems_every_entry_point(seed):
    """Shapes, m, lambda, solve counts, outliers drawn at random; the entry point or option under
    test cycles with the seed.  Each result against the oracle's routine for that entry point."""
    from paper_2302_05865_amd import fa_aggregate_static
    rng = np.random.default_rng(70_000 + seed)
    kind = _ENTRY_KINDS[seed % len(_ENTRY_KINDS)]
    p = int(rng.integers(2, 65))
    m = int(rng.integers(1, p + 1))
    lam = float(rng.choice([0.0, 0.3, 1.0, 4.0]))
    iters = int(rng.integers(1, 13))
    n = int(rng.integers(p + 1, 5000))
    announce("random entry", seed, kind, p, m, lam, iters, n)
    mu = rng.standard_normal(n)
    G32 = (mu[None, :] * rng.uniform(0.2, 2.0, p)[:, None] +
           rng.uniform(0.05, 1.5) * rng.standard_normal((p, n))).astype(np.float32)
    for b in rng.choice(p, size=int(rng.integers(0, max(1, p // 4) + 1)), replace=False):
        G32[b] = (-4.0 * mu if rng.random() < 0.5 else 30.0 * rng.standard_normal(n)).astype(np.float32)
    bf = kind in ("bf16", "row_major_bf16") or (kind in ("static", "arrival", "krum") and rng.random() < 0.4)
    Gw = si.f32_to_bf16_bits(G32.reshape(-1)).reshape(p, n) if bf else G32
    dt = "bf16" if bf else "f32"
    info = None
    if kind in ("bf16", "stop_rule"):
        tol = 0.0 if kind == "bf16" else float(rng.choice([1e-3, 1e-5]))
        ref = fa_scaled(Gw, m, lam, iters, tol)
        agg = FlagAggregator(n_max=n, p_max=p, dtype=dt)
        out = agg.fa_aggregate(to_device(Gw), m, lam, iters, tol)
        info = agg.fa_get_info()
        assert info.iters_done == ref["iters_done"]
    elif kind in ("row_major", "row_major_bf16"):
        es = 2 if bf else 4
        pitch = ((p * es + 15) // 16) * 16 // es
        ref = fa_scaled(Gw, m, lam, iters, 0.0)
        agg = FlagAggregator(n_max=n, p_max=p, dtype=dt, layout="row_major")
        out = agg.fa_aggregate(_rows_device(Gw, pitch), m, lam, iters, 0.0)
        info = agg.fa_get_info()
    elif kind == "exponent":
        a = float(rng.choice([1.0, 1.5, 3.0, 6.0]))
        ref = fa_scaled(Gw, m, lam, iters, 0.0, a=a)
        agg = FlagAggregator(n_max=n, p_max=p, exponent_a=a)
        out = agg.fa_aggregate(to_device(Gw), m, lam, iters, 0.0)
        info = agg.fa_get_info()
    elif kind == "restream":
        ref = fa_scaled(Gw, m, lam, iters, 0.0)
        agg = FlagAggregator(n_max=n, p_max=p)
        out = agg.fa_aggregate_restream(to_device(Gw), m, lam, iters)
        info = agg.fa_get_info()
    elif kind == "static":
        agg = None
        ref = fa_scaled(Gw, m, lam, iters, 0.0)
        out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        fa_aggregate_static(to_device(Gw), m, lam, iters, 0.0, out)
    elif kind == "arrival":
        ref = fa_scaled(Gw, m, lam, iters, 0.0)
        agg = FlagAggregator(n_max=n, p_max=p, dtype=dt)
        full, buf = to_device(Gw), to_device(np.zeros_like(Gw))
        agg.fa_gram_begin(p, n)
        for i in rng.permutation(p):
            buf[i] = full[i]
            agg.fa_gram_update(buf, int(i))
        out = agg.fa_aggregate_arrived(buf, m, lam, iters, 0.0)
        info = agg.fa_get_info()
    elif kind == "krum":
        f = min(int(rng.integers(0, max(1, p - 2))), max(p - 3, 0))
        q = int(rng.integers(1, p + 1))
        if p - f - 2 < 1:
            pytest.skip("Multi-Krum needs p - f - 2 >= 1")
        ref = multi_krum(as_f64_matrix(Gw), f, q)
        agg = FlagAggregator(n_max=n, p_max=p, dtype=dt)
        out, scores, sel = agg.fa_multikrum(to_device(Gw), f, q)
        sc = np.sort(ref["scores"])
        if q == p or (sc[q] - sc[q - 1]) > 1e-9 * sc[-1]:      # no near-tie at the cut
            assert np.array_equal(sel, ref["selected"])
        else:
            ref = None
    else:   # grouped
        nw = int(rng.integers(1, min(p, 8) + 1))
        cuts = np.sort(rng.choice(np.arange(1, p), size=nw - 1, replace=False)) if nw > 1 else []
        sizes = np.diff(np.concatenate([[0], cuts, [p]])).astype(int).tolist()
        ref = fa_literal_grouped(as_f64_matrix(Gw), sizes, m, lam, iters, 0.0)
        agg = FlagAggregator(n_max=n, p_max=p)
        out = agg.fa_aggregate_grouped(to_device(Gw), sizes, m, lam, iters, 0.0)
    if ref is not None:
        assert rel_l2(out.cpu().numpy().astype(np.float64), ref["out"]) <= GATE
        if info is not None:
            assert info.status == 0
            assert projector_difference(info.A, ref["A"], ref["R"]) <= GATE
    if agg is not None:
        agg.close()
