"""Pins for the CPU oracle: what the paper and the mathematics fix about the Flag
Aggregator, checked without reference to the oracle's own formulas.

Each test names the statement of the paper it rests on.  None of them needs a GPU.
"""
import math

import numpy as np
import pytest

from oracle import (as_f64_matrix, basis_products, decode_bf16, fa_literal, fa_literal_grouped,
                    fa_scaled, multi_krum, projector_difference, tsqr_r)


def _rand(n, p, seed, col_scales=True):
    rng = np.random.default_rng(seed)
    G = rng.standard_normal((n, p))
    if col_scales:
        G = G * rng.uniform(0.3, 4.0, p)[None, :]
    return G


def _principal_cosines(Y1, Y2):
    return np.linalg.svd(Y1.T @ Y2, compute_uv=False)


# Independent statement of the FA objective (Eq. 5 + Sec. 2.3 option (2)), with explicit
# loops over workers and over ordered pairs i != j.
def eq5_objective(Y, G, lam, pair_factor=None, a=2.0):
    n, p = G.shape
    total = 0.0
    for i in range(p):
        g = G[:, i]
        z = Y.T @ g
        total += max(1.0 - float(z @ z) / float(g @ g), 0.0) ** (1.0 / a)
    if lam > 0:
        fac = lam / (p - 1) if pair_factor is None else pair_factor
        for i in range(p):
            for j in range(p):
                if i == j:
                    continue
                d = G[:, i] - G[:, j]
                z = Y.T @ d
                total += fac * max(1.0 - float(z @ z) / float(d @ d), 0.0) ** (1.0 / a)
    return total


def _retract(Y, D, t):
    Q, R = np.linalg.qr(Y + t * D)
    return Q * np.sign(np.diag(R))[None, :]


# --------------------------------------------------------------------------- PCA pin
@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("m", [1, 3, 5])
def test_first_solve_is_pca(seed, m):
    """Appendix E.2: one FA iteration with uniform weights is PCA of the (normalised)
    gradient matrix.  Reference route: eigenvectors of the n x n matrix sum_i g~_i g~_i^T."""
    G = _rand(30, 7, seed)
    res = fa_literal(G, m, 0.0, 1, 0.0)
    Gn = G / np.linalg.norm(G, axis=0)[None, :]
    evals, evecs = np.linalg.eigh(Gn @ Gn.T)
    top = evecs[:, np.argsort(-evals)[:m]]
    cos = _principal_cosines(top, res["Y"])
    assert np.all(np.abs(cos - 1.0) < 1e-10)
    # the output is the column average of the reconstruction Y Y^T G (Sec. 2.1, Alg. 1)
    recon = top @ (top.T @ G)
    assert np.allclose(res["out"], recon.mean(axis=1), rtol=0, atol=1e-10 * np.abs(G).max())


@pytest.mark.parametrize("lam", [0.0, 0.7])
def test_feasibility_and_ratio_range(lam):
    """Eq. 5 constraint Y^T Y = I; Sec. 2.1/2.2: explained variances lie in [0, 1]."""
    G = _rand(25, 9, 3)
    res = fa_literal(G, 4, lam, 7, 0.0)
    Y = res["Y"]
    assert np.abs(Y.T @ Y - np.eye(4)).max() < 1e-12
    assert np.all(res["v"] >= 0) and np.all(res["v"] <= 1 + 1e-12)
    assert np.all(res["u"] >= 0) and np.all(res["u"] <= 1 + 1e-12)
    # the ratios really are ||Y^T g||^2 / ||g||^2
    for i in range(9):
        g = G[:, i]
        assert abs(res["v"][i] - np.sum((Y.T @ g) ** 2) / (g @ g)) < 1e-12


@pytest.mark.parametrize("lam", [0.0, 1.0, 10.0])
@pytest.mark.parametrize("iters", [1, 6])
def test_full_subspace_gives_the_mean(lam, iters):
    """Sec. 2.1: g in span(Y) is fully explained and Y Y^T G reconstructs G, so with
    m >= rank(G) the aggregate is the plain mean of the gradients and all ratios are 1."""
    G = _rand(20, 6, 4)
    res = fa_literal(G, 6, lam, iters, 0.0)
    assert np.allclose(res["out"], G.mean(axis=1), atol=1e-12 * np.abs(G).max() * 10)
    assert np.allclose(res["v"], 1.0, atol=1e-12)
    # rank-deficient G (rank 3) with m = 3 < p
    rng = np.random.default_rng(9)
    B = rng.standard_normal((20, 3))
    G3 = B @ rng.standard_normal((3, 6))
    res = fa_literal(G3, 3, lam, iters, 0.0)
    assert np.allclose(res["out"], G3.mean(axis=1), atol=1e-11 * np.abs(G3).max())
    assert np.allclose(res["v"], 1.0, atol=1e-11)


@pytest.mark.parametrize("lam", [0.0, 1.0])
@pytest.mark.parametrize("m", [1, 3])
def test_identical_gradients(lam, m):
    """All workers send the same g: the aggregate must be g (rank 1; with lam > 0 every
    pairwise distance D_ij is zero and those terms drop out)."""
    g = np.random.default_rng(5).standard_normal(17)
    G = np.repeat(g[:, None], 5, axis=1)
    res = fa_literal(G, m, lam, 4, 0.0)
    assert np.allclose(res["out"], g, atol=1e-12)
    res_s = fa_scaled(np.ascontiguousarray(G.T), m, lam, 4, 0.0)
    assert np.allclose(res_s["out"], g, atol=1e-12)


@pytest.mark.parametrize("theta_deg", [20.0, 60.0, 85.0])
def test_two_workers_bisector(theta_deg):
    """p = 2, m = 1, lam = 0: PCA of two unit directions at an acute angle is their
    bisector; by symmetry the two ratios (hence weights) stay equal, so every IRLS solve
    returns the bisector again.  Ratios equal cos^2(theta/2)."""
    th = math.radians(theta_deg)
    n = 6
    rng = np.random.default_rng(11)
    Q, _ = np.linalg.qr(rng.standard_normal((n, 2)))
    a = Q[:, 0]
    b = math.cos(th) * Q[:, 0] + math.sin(th) * Q[:, 1]
    G = np.stack([2.5 * a, 0.4 * b], axis=1)          # different norms
    res = fa_literal(G, 1, 0.0, 9, 0.0)
    y = (a + b) / np.linalg.norm(a + b)
    assert abs(abs(float(y @ res["Y"][:, 0])) - 1.0) < 1e-12
    assert np.allclose(res["v"], math.cos(th / 2) ** 2, atol=1e-12)
    expect = 0.5 * y * float(y @ (G[:, 0] + G[:, 1]))
    assert np.allclose(res["out"], expect, atol=1e-12)
    # objective trace: 2 sin(theta/2) at every solve
    assert np.allclose(res["objective"], 2 * math.sin(th / 2), atol=1e-10)


def test_orthogonal_columns_total_tie():
    """Mutually orthogonal gradients, lam = 0: the normalised Gram matrix is the identity
    and every m-dimensional subspace of span(G) is a valid first solve.  What is unique:
    Y^T Y = I, Y in span(G), and sum_i v_i = m."""
    rng = np.random.default_rng(2)
    Q, _ = np.linalg.qr(rng.standard_normal((15, 6)))
    G = Q * rng.uniform(0.5, 2.0, 6)[None, :]
    res = fa_literal(G, 3, 0.0, 1, 0.0)
    Y = res["Y"]
    assert np.abs(Y.T @ Y - np.eye(3)).max() < 1e-12
    assert np.linalg.norm(Y - Q @ (Q.T @ Y)) < 1e-12
    assert abs(res["v"].sum() - 3.0) < 1e-12


# ----------------------------------------------------------------- IRLS as MM procedure
@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("lam", [0.0, 1.0])
def test_objective_monotone_while_unclamped(seed, lam):
    """Appendix E.2 / Sec. 2.3: the re-weighting is a convergent procedure; as a
    majorise-minimise scheme for Eq. 5 the objective cannot rise (weight floor inactive)."""
    G = _rand(14, 8, 20 + seed)
    p, delta = 8, 1e-6
    off = ~np.eye(p, dtype=bool)
    prev = None
    checked = 0
    for k in range(1, 31):
        res = fa_literal(G, 2, lam, k, 0.0, delta=delta)
        obj = res["objective"][-1]
        # the recorded objective equals Eq. 5 evaluated independently at this Y
        assert abs(obj - eq5_objective(res["Y"], G, lam)) < 1e-7
        if prev is not None and prev[1] > delta:      # floor was inactive for this step
            assert obj <= prev[0] + 1e-10
            checked += 1
        min_rho = (1 - res["v"]).min()
        if lam > 0:
            min_rho = min(min_rho, (1 - res["u"][off]).min())
        prev = (obj, min_rho)
    assert checked >= 3


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_converged_point_is_stationary_for_eq5(seed):
    """The fixed point of the IRLS must be a stationary point of Eq. 5 itself (objective
    written out independently above, ordered pairs, factor lam/(p-1)).  This pins the
    weight exponent (-1/2 on the residual), the pairwise normalisation by D_ij and the
    ordered-pair factor: with any of them changed the fixed point moves and the
    derivative below is O(0.1)."""
    rng = np.random.default_rng(seed)
    n, p, m, lam = 12, 8, 2, 1.0
    G = rng.standard_normal((n, p)) * rng.uniform(0.5, 3, p)[None, :]
    res = fa_literal(G, m, lam, 400, 0.0)
    Y = res["Y"]
    off = ~np.eye(p, dtype=bool)
    assert min((1 - res["v"]).min(), (1 - res["u"][off]).min()) > 1e-3   # interior point
    worst = 0.0
    worst_wrong_factor = 0.0
    h = 1e-5
    for _ in range(6):
        D = rng.standard_normal((n, m))
        D -= Y @ (Y.T @ D)
        D /= np.linalg.norm(D)
        dd = (eq5_objective(_retract(Y, D, h), G, lam)
              - eq5_objective(_retract(Y, D, -h), G, lam)) / (2 * h)
        worst = max(worst, abs(dd))
        fac = 0.5 * lam / (p - 1)        # what an unordered pair sum would give
        dw = (eq5_objective(_retract(Y, D, h), G, lam, fac)
              - eq5_objective(_retract(Y, D, -h), G, lam, fac)) / (2 * h)
        worst_wrong_factor = max(worst_wrong_factor, abs(dw))
    assert worst < 1e-6
    assert worst_wrong_factor > 1e-3      # the check has power


def eq5_floored(Y, G, lam, a, delta):
    """Eq. 5 with exponent 1/a (Sec. 2.2, Step 2) and every term continued linearly below the
    floor: phi(rho) = rho^(1/a) for rho >= delta, and its tangent at delta below.  This is the
    function whose slope is the floored IRLS weight max(rho, delta)^(1/a - 1) / a, so a fixed
    point of the floored IRLS must be a stationary point of it, vertex or not (Appendix D
    perturbs the root for the same purpose)."""
    def phi(rho):
        rho = max(rho, 0.0)
        if rho >= delta:
            return rho ** (1.0 / a)
        return delta ** (1.0 / a) + (rho - delta) * delta ** (1.0 / a - 1.0) / a
    n, p = G.shape
    total = 0.0
    for i in range(p):
        g = G[:, i]
        z = Y.T @ g
        total += phi(1.0 - float(z @ z) / float(g @ g))
    if lam > 0:
        for i in range(p):
            for j in range(p):
                if i != j:
                    d = G[:, i] - G[:, j]
                    z = Y.T @ d
                    total += lam / (p - 1) * phi(1.0 - float(z @ z) / float(d @ d))
    return total


@pytest.mark.parametrize("a,seed", [(1.5, 1), (1.5, 2), (3.0, 1), (3.0, 20), (4.0, 20)])
def test_general_exponent_interior_fixed_point_is_stationary(seed, a):
    """Sec. 2.2, Step 2: with the Taylor constant a every term is (1 - v)^(1/a).  An IRLS
    fixed point away from every vertex must be stationary for that objective (written out
    independently), and not for another exponent's: pins the weight exponent 1/a - 1.
    (The inputs are the ones of this recipe that converge to an interior point; the floored
    variant below covers the vertex solutions that large a prefers.)"""
    rng = np.random.default_rng(seed)
    n, p, m, lam = 12, 8, 2, 1.0
    G = rng.standard_normal((n, p)) * rng.uniform(0.5, 3, p)[None, :]
    res = fa_literal(G, m, lam, 1500, 0.0, a=a)
    Y = res["Y"]
    off = ~np.eye(p, dtype=bool)
    assert min((1 - res["v"]).min(), (1 - res["u"][off]).min()) > 1e-3    # interior
    assert abs(res["objective"][-1] - eq5_objective(Y, G, lam, a=a)) < 1e-7
    worst = worst_other = 0.0
    h = 1e-5
    other = 2.0 if a != 2.0 else 3.0
    for _ in range(6):
        D = rng.standard_normal((n, m))
        D -= Y @ (Y.T @ D)
        D /= np.linalg.norm(D)
        dd = (eq5_objective(_retract(Y, D, h), G, lam, a=a)
              - eq5_objective(_retract(Y, D, -h), G, lam, a=a)) / (2 * h)
        worst = max(worst, abs(dd))
        do = (eq5_objective(_retract(Y, D, h), G, lam, a=other)
              - eq5_objective(_retract(Y, D, -h), G, lam, a=other)) / (2 * h)
        worst_other = max(worst_other, abs(do))
    assert worst < 1e-5
    assert worst_other > 1e-3


@pytest.mark.parametrize("a", [1.5, 2.0, 3.0, 4.0, 6.0])
@pytest.mark.parametrize("seed", [1, 2])
def test_floored_irls_fixed_point_is_stationary_for_the_floored_objective(seed, a):
    """The floor makes the IRLS a majorise-minimise scheme for Eq. 5 with every term continued
    by its tangent below delta (eq5_floored): its fixed points are stationary points of that
    smooth function also where gradients are explained exactly, which is where the iteration
    ends up for large a.  Pins, for every exponent used anywhere (2, the GPU tests' 4, and 6):
    the weight exponent, that the floor acts on the residual, and the ordered-pair factor."""
    rng = np.random.default_rng(seed)
    n, p, m, lam, delta = 12, 8, 2, 1.0, 0.05
    G = rng.standard_normal((n, p)) * rng.uniform(0.5, 3, p)[None, :]
    res = fa_literal(G, m, lam, 4000, 0.0, delta=delta, a=a)
    Y = res["Y"]
    worst = worst_other = worst_floor = 0.0
    h = 1e-5
    other = 2.0 if a != 2.0 else 4.0
    for _ in range(6):
        D = rng.standard_normal((n, m))
        D -= Y @ (Y.T @ D)
        D /= np.linalg.norm(D)
        Yp, Ym = _retract(Y, D, h), _retract(Y, D, -h)
        worst = max(worst, abs(eq5_floored(Yp, G, lam, a, delta)
                               - eq5_floored(Ym, G, lam, a, delta)) / (2 * h))
        worst_other = max(worst_other, abs(eq5_floored(Yp, G, lam, other, delta)
                                           - eq5_floored(Ym, G, lam, other, delta)) / (2 * h))
        worst_floor = max(worst_floor, abs(eq5_floored(Yp, G, lam, a, delta / 50)
                                           - eq5_floored(Ym, G, lam, a, delta / 50)) / (2 * h))
    assert worst < 1e-6
    assert worst_other > 1e-3          # another exponent's objective is not stationary here
    assert worst_floor > 1e-3 or (1 - res["v"]).min() > delta   # nor is another floor's


def test_exponent_one_is_pca_whatever_the_iteration_count():
    """a = 1 makes every term linear in its residual: the weights never move, and every
    solve is the first one (weighted PCA with unit weights)."""
    G = _rand(15, 6, 77)
    first = fa_literal(G, 3, 1.0, 1, 0.0)
    many = fa_literal(G, 3, 1.0, 9, 0.0, a=1.0)
    assert np.allclose(many["Y"] @ many["Y"].T, first["Y"] @ first["Y"].T, atol=1e-10)
    assert np.allclose(many["w"], 1.0) and np.allclose(many["out"], first["out"], atol=1e-10)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("lam", [0.0, 1.0])
def test_converged_point_is_a_local_minimum_by_sampling(seed, lam):
    """Brute force: no nearby feasible Y has a lower Eq. 5 value than the converged one
    (also at 'vertex' solutions where some gradients are explained exactly)."""
    rng = np.random.default_rng(100 + seed)
    n, p, m = 9, 7, 2
    G = rng.standard_normal((n, p)) * rng.uniform(0.5, 3, p)[None, :]
    # a small weight floor, so that the fixed point sits within ~sqrt(delta) of the vertex
    res = fa_literal(G, m, lam, 500, 0.0, delta=1e-12)
    Y = res["Y"]
    a0 = eq5_objective(Y, G, lam)
    for _ in range(300):
        D = rng.standard_normal((n, m))
        t = 10 ** rng.uniform(-4, -1.5)
        assert eq5_objective(_retract(Y, D, t), G, lam) >= a0 - 2e-5


def test_iters_and_tol_semantics():
    """Sec. 3 'Implementation Details': stop at a small error or after a fixed number of
    flag-mean solves.  iters counts solves; tol compares successive objective values."""
    G = _rand(16, 7, 7)
    full = fa_literal(G, 3, 1.0, 30, 0.0)
    assert full["iters_done"] == 30
    tol = 1e-3
    early = fa_literal(G, 3, 1.0, 30, tol)
    obj = np.array(full["objective"])
    k_stop = next(k for k in range(1, 30) if abs(obj[k - 1] - obj[k]) < tol)
    assert early["iters_done"] == k_stop + 1
    ref = fa_literal(G, 3, 1.0, k_stop + 1, 0.0)
    assert np.allclose(early["out"], ref["out"], atol=1e-14)
    # the test needs two objective values: a huge tol stops right after the second solve
    assert fa_literal(G, 3, 1.0, 30, 1e9)["iters_done"] == 2
    assert fa_literal(G, 3, 1.0, 1, 1e9)["iters_done"] == 1


def test_weight_floor_is_applied():
    """Readings: weights are max(rho, delta)^(-1/2); an exactly explained worker gets
    delta^(-1/2)."""
    G = _rand(10, 4, 8)
    res = fa_literal(G, 2, 0.0, 60, 0.0, delta=1e-6)
    assert res["w"].max() <= 1e3 * (1 + 1e-12)
    rho = 1 - res["v"]
    expect = np.maximum(rho, 1e-6) ** -0.5
    assert np.allclose(res["w"], expect, rtol=1e-6)


# ------------------------------------------------------------------------ metamorphic
@pytest.mark.parametrize("lam", [0.0, 1.0])
def test_permutation_scale_rotation(lam):
    G = _rand(18, 7, 12)
    m, iters = 3, 6
    base = fa_literal(G, m, lam, iters, 0.0)
    rng = np.random.default_rng(0)
    perm = rng.permutation(7)
    r = fa_literal(G[:, perm], m, lam, iters, 0.0)
    assert np.allclose(r["out"], base["out"], atol=1e-10)
    assert np.allclose(r["v"], base["v"][perm], atol=1e-10)
    r = fa_literal(-3.5 * G, m, lam, iters, 0.0)
    assert np.allclose(r["out"], -3.5 * base["out"], atol=1e-10)
    Q, _ = np.linalg.qr(rng.standard_normal((18, 18)))
    r = fa_literal(Q @ G, m, lam, iters, 0.0)
    assert np.allclose(r["out"], Q @ base["out"], atol=1e-10)
    # output lies in span(G) (Appendix D: Y Y^T G = G S_FA + ...)
    coef, *_ = np.linalg.lstsq(G, base["out"], rcond=None)
    assert np.linalg.norm(G @ coef - base["out"]) < 1e-10


def test_column_rescaling_leaves_subspace_unchanged_at_lambda0():
    """At lam = 0 only the normalised gradients enter Eq. 5, so positive per-column
    rescaling leaves Y (and the ratios) unchanged."""
    G = _rand(18, 7, 13)
    a = fa_literal(G, 3, 0.0, 8, 0.0)
    alpha = np.random.default_rng(1).uniform(0.1, 9.0, 7)
    b = fa_literal(G * alpha[None, :], 3, 0.0, 8, 0.0)
    assert np.all(np.abs(_principal_cosines(a["Y"], b["Y"]) - 1) < 1e-10)
    assert np.allclose(a["v"], b["v"], atol=1e-10)


def test_zero_column_is_a_dropped_worker():
    """A zero gradient (a worker whose message was lost and zeroed at the server, Sec. 3
    communication-loss experiment) has no direction: at lam = 0 the subspace is that of
    the remaining workers and the aggregate scales by (p-1)/p."""
    G = _rand(15, 6, 14)
    Gz = np.concatenate([G[:, :2], np.zeros((15, 1)), G[:, 2:]], axis=1)
    a = fa_literal(G, 2, 0.0, 5, 0.0)
    b = fa_literal(Gz, 2, 0.0, 5, 0.0)
    assert np.allclose(b["out"], a["out"] * 6 / 7, atol=1e-12)
    assert b["w"][2] == 0.0 and b["v"][2] == 0.0
    # with lam > 0 the call must still be finite
    c = fa_literal(Gz, 2, 1.0, 5, 0.0)
    assert np.all(np.isfinite(c["out"]))


def test_lambda_large_pairs_dominate():
    """Sec. 2.3: with lam = Theta(p) the pairwise terms dominate.  As lam grows the first
    solve tends to PCA of the normalised pairwise differences alone."""
    G = _rand(16, 6, 15)
    p = 6
    diffs = []
    for i in range(p):
        for j in range(p):
            if i != j:
                d = G[:, i] - G[:, j]
                diffs.append(d / np.linalg.norm(d))
    Dn = np.stack(diffs, axis=1)
    evals, evecs = np.linalg.eigh(Dn @ Dn.T)
    top = evecs[:, np.argsort(-evals)[:2]]
    r = fa_literal(G, 2, 1e9, 1, 0.0)
    assert np.all(np.abs(_principal_cosines(top, r["Y"]) - 1) < 1e-7)


# -------------------------------------------------------------- scaled form == literal
@pytest.mark.parametrize("lam", [0.0, 0.1, 1.0])
@pytest.mark.parametrize("shape", [(200, 8, 4), (97, 5, 2), (64, 3, 3)])
def test_scaled_matches_literal(lam, shape):
    n, p, m = shape
    G = _rand(n, p, n + p)
    Gw = np.ascontiguousarray(G.T)
    a = fa_literal(G, m, lam, 9, 0.0)
    b = fa_scaled(Gw, m, lam, 9, 0.0, chunk_rows=37)
    assert np.linalg.norm(a["out"] - b["out"]) <= 1e-11 * np.linalg.norm(a["out"])
    assert np.allclose(a["v"], b["v"], atol=1e-11)
    assert np.allclose(a["objective"], b["objective"], atol=1e-6)   # sqrt of 1e-16 noise at exact fits
    # Y = G A reproduces the literal subspace
    Yb = G @ b["A"]
    assert np.abs(Yb.T @ Yb - np.eye(m)).max() < 1e-10
    assert np.all(np.abs(_principal_cosines(a["Y"], Yb) - 1) < 1e-10)
    K = G.T @ G
    assert np.allclose(b["K"], K, atol=1e-10 * np.abs(K).max())
    assert projector_difference(b["A"], b["A"], b["R"]) == 0.0


def test_tsqr_is_an_isometry_with_duplicates_and_ragged_chunks():
    rng = np.random.default_rng(3)
    Gw = rng.standard_normal((5, 1003)).astype(np.float32)
    Gw[3] = Gw[1]                                 # exact duplicate column
    R = tsqr_r(Gw, chunk_rows=100)
    G = as_f64_matrix(Gw)
    assert np.allclose(R.T @ R, G.T @ G, atol=1e-9)
    assert np.allclose(np.tril(R, -1), 0.0)
    res = fa_scaled(Gw, 2, 1.0, 5, 0.0, chunk_rows=100)
    lit = fa_literal(G, 2, 1.0, 5, 0.0)
    assert np.linalg.norm(res["out"] - lit["out"]) <= 1e-10 * np.linalg.norm(lit["out"])


def test_projector_difference_matches_dense():
    rng = np.random.default_rng(4)
    G = rng.standard_normal((30, 5))
    A1 = rng.standard_normal((5, 2))
    A2 = rng.standard_normal((5, 2))
    P1 = (G @ A1) @ (G @ A1).T
    P2 = (G @ A2) @ (G @ A2).T
    R = np.linalg.qr(G, mode="r")
    assert abs(projector_difference(A1, A2, R) - np.linalg.norm(P1 - P2)) < 1e-9
    # linearly dependent gradients: null-space components of A must not register
    G2 = np.concatenate([G, G[:, :1]], axis=1)
    R2 = np.linalg.qr(G2, mode="r")
    B1 = np.concatenate([A1, np.zeros((1, 2))], axis=0)
    B2 = B1.copy()
    B2[0] += 0.5
    B2[5] -= 0.5                      # same G2 @ B, different representation
    assert projector_difference(B1, B2, R2) < 1e-12


# ---- workers that send several gradients (blocks of columns) ------------------------------------
def _grouped_objective(Y, G, sizes, lam):
    """Eq. 5 with blocks, written out independently: values tr(g^T Y Y^T g) / tr(g^T g),
    pair terms only between blocks of equal width, factor lam / (P - 1), ordered pairs."""
    off = np.concatenate([[0], np.cumsum(sizes)])
    B = [G[:, off[i]:off[i + 1]] for i in range(len(sizes))]
    tot = 0.0
    for b in B:
        tot += math.sqrt(max(1.0 - np.sum((Y.T @ b) ** 2) / np.sum(b * b), 0.0))
    P = len(B)
    for i in range(P):
        for j in range(P):
            if i != j and sizes[i] == sizes[j]:
                d = B[i] - B[j]
                tot += lam / (P - 1) * math.sqrt(max(1.0 - np.sum((Y.T @ d) ** 2) / np.sum(d * d), 0.0))
    return tot


@pytest.mark.parametrize("lam", [0.0, 1.0])
def test_grouped_with_single_columns_is_the_plain_method(lam):
    G = _rand(30, 6, 5)
    a = fa_literal(G, 3, lam, 7, 0.0)
    b = fa_literal_grouped(G, [1] * 6, 3, lam, 7, 0.0)
    assert np.allclose(a["out"], b["out"], atol=1e-12)
    assert np.allclose(a["v"], b["v"], atol=1e-12)
    assert np.allclose(a["objective"], b["objective"], atol=1e-12)


def test_grouped_repeated_gradient_counts_once():
    """A worker that sends the same gradient k times is the worker that sends it once (no
    pair terms: they only exist between blocks of equal width)."""
    G = _rand(40, 5, 8)
    sizes = [3, 1, 2, 1, 4]
    Gg = np.concatenate([np.repeat(G[:, i:i + 1], k, axis=1) for i, k in enumerate(sizes)], axis=1)
    a = fa_literal(G, 2, 0.0, 9, 0.0)
    b = fa_literal_grouped(Gg, sizes, 2, 0.0, 9, 0.0)
    assert np.allclose(a["out"], b["out"], atol=1e-11)
    assert np.allclose(a["v"], b["v"], atol=1e-11)
    assert np.allclose(a["objective"], b["objective"], atol=1e-11)


def test_grouped_value_ignores_a_rotation_within_a_block():
    rng = np.random.default_rng(2)
    G = _rand(35, 7, 9)
    sizes = [3, 2, 2]
    Q = np.linalg.qr(rng.standard_normal((3, 3)))[0]
    G2 = G.copy()
    G2[:, :3] = G[:, :3] @ Q
    a = fa_literal_grouped(G, sizes, 2, 0.0, 6, 0.0)
    b = fa_literal_grouped(G2, sizes, 2, 0.0, 6, 0.0)
    assert np.allclose(a["v"], b["v"], atol=1e-11)
    assert np.allclose(a["objective"], b["objective"], atol=1e-11)
    assert np.allclose(a["Y"] @ a["Y"].T, b["Y"] @ b["Y"].T, atol=1e-9)


@pytest.mark.parametrize("seed", [0, 1])
def test_grouped_fixed_point_is_stationary(seed):
    """As for Eq. 5 itself: the fixed point of the block IRLS is a stationary point of the
    block objective written out above (pins the block normalisation, which pairs exist,
    and the factor lam / (P - 1))."""
    rng = np.random.default_rng(seed)
    n, sizes, m, lam = 20, [3, 3, 4, 3, 3], 2, 1.0    # blocks wider than m: interior point
    G = rng.standard_normal((n, sum(sizes))) * rng.uniform(0.5, 3, sum(sizes))[None, :]
    res = fa_literal_grouped(G, sizes, m, lam, 500, 0.0)
    Y = res["Y"]
    assert (1 - res["v"]).min() > 1e-3
    worst = worst_wrong = 0.0
    h = 1e-5
    for _ in range(6):
        D = rng.standard_normal((n, m))
        D -= Y @ (Y.T @ D)
        D /= np.linalg.norm(D)
        dd = (_grouped_objective(_retract(Y, D, h), G, sizes, lam)
              - _grouped_objective(_retract(Y, D, -h), G, sizes, lam)) / (2 * h)
        worst = max(worst, abs(dd))
        dw = (_grouped_objective(_retract(Y, D, h), G, sizes, 3 * lam)
              - _grouped_objective(_retract(Y, D, -h), G, sizes, 3 * lam)) / (2 * h)
        worst_wrong = max(worst_wrong, abs(dw))
    assert worst < 1e-6
    assert worst_wrong > 1e-3


def test_grouped_output_is_the_projected_mean_of_worker_means():
    G = _rand(25, 6, 4)
    sizes = [2, 3, 1]
    res = fa_literal_grouped(G, sizes, 6, 1.0, 3, 0.0)          # m = all columns: Y spans G
    gbar = (G[:, :2].mean(axis=1) + G[:, 2:5].mean(axis=1) + G[:, 5]) / 3
    assert np.allclose(res["out"], gbar, atol=1e-10)


# ---- Multi-Krum (the comparison aggregator that shares the Gram matrix) -------------------------
def test_multi_krum_worked_example_on_a_line():
    """Five workers on a line at 0, 1, 2, 3 and 10 (one coordinate), f = 1: each is scored by its
    p - f - 2 = 2 nearest.  Squared distances by hand: worker 0: {1, 4}; 1: {1, 1}; 2: {1, 1};
    3: {1, 4}; 4 (the outlier): {49, 64}."""
    G = np.array([[0.0, 1.0, 2.0, 3.0, 10.0]])
    res = multi_krum(G, 1, 2)
    assert np.array_equal(res["scores"], [5.0, 2.0, 2.0, 5.0, 113.0])
    assert np.array_equal(res["selected"], [0, 1, 1, 0, 0])          # the two best; ties by index
    assert np.allclose(res["out"], [1.5])
    res = multi_krum(G, 1, 4)                                         # p - f of them: all but the outlier
    assert np.array_equal(res["selected"], [1, 1, 1, 1, 0]) and np.allclose(res["out"], [1.5])
    res = multi_krum(G, 1, 3)                                         # tie 0 / 3 goes to the smaller index
    assert np.array_equal(res["selected"], [1, 1, 1, 0, 0])


def test_multi_krum_properties():
    rng = np.random.default_rng(6)
    G = rng.standard_normal((30, 9))
    G[:, 7] = 50.0 * rng.standard_normal(30)          # two far outliers
    G[:, 2] = -20.0 * G[:, 0]
    res = multi_krum(G, 2, 7)
    assert res["selected"][7] == 0 and res["selected"][2] == 0 and res["selected"].sum() == 7
    keep = [i for i in range(9) if i not in (2, 7)]
    assert np.allclose(res["out"], G[:, keep].mean(axis=1))
    # selecting everybody is the mean; a permutation of the workers permutes the scores
    assert np.allclose(multi_krum(G, 0, 9)["out"], G.mean(axis=1))
    perm = rng.permutation(9)
    assert np.allclose(multi_krum(G[:, perm], 2, 7)["scores"], res["scores"][perm])
    # a rotation of the coordinates changes no distance
    Q = np.linalg.qr(rng.standard_normal((30, 30)))[0]
    assert np.allclose(multi_krum(Q @ G, 2, 7)["scores"], res["scores"], rtol=1e-10)
    with pytest.raises(ValueError):
        multi_krum(G, 7, 2)


def test_basis_products_by_brute_force_and_on_a_solution():
    # entry by entry, with plain loops
    rng = np.random.default_rng(11)
    G = rng.standard_normal((9, 4))
    Y = rng.standard_normal((9, 3))
    YtY, YtG = basis_products(G, Y)
    for a in range(3):
        for b in range(3):
            assert math.isclose(YtY[a, b], sum(Y[k, a] * Y[k, b] for k in range(9)),
                                rel_tol=1e-12, abs_tol=1e-14)
        for i in range(4):
            assert math.isclose(YtG[a, i], sum(Y[k, a] * G[k, i] for k in range(9)),
                                rel_tol=1e-12, abs_tol=1e-14)
    # an orthonormal basis gives the identity; a transposed operand would not even have the shape
    Q = np.linalg.qr(rng.standard_normal((40, 5)))[0]
    I5, QtG = basis_products(rng.standard_normal((40, 7)), Q)
    assert I5.shape == (5, 5) and QtG.shape == (5, 7) and np.allclose(I5, np.eye(5), atol=1e-13)
    # on a solution of the method the column sums of squares of Y^T G are the explained variances
    G = _rand(60, 6, 3)
    res = fa_literal(G, 3, 1.0, 5, 0.0)
    YtY, YtG = basis_products(G, res["Y"])
    assert np.allclose(YtY, np.eye(3), atol=1e-12)
    assert np.allclose((YtG ** 2).sum(axis=0) / (G ** 2).sum(axis=0), res["v"], atol=1e-12)


def test_bf16_decode_known_patterns():
    bits = np.array([0x3F80, 0xC000, 0x3FC0, 0x0000, 0x8000, 0x7F80], dtype=np.uint16)
    vals = decode_bf16(bits)
    assert vals.dtype == np.float32
    assert vals[0] == 1.0 and vals[1] == -2.0 and vals[2] == 1.5
    assert vals[3] == 0.0 and np.signbit(vals[4]) and np.isinf(vals[5])


def test_argument_errors():
    G = _rand(10, 4, 1)
    with pytest.raises(ValueError):
        fa_literal(G, 0, 0.0, 1, 0.0)
    with pytest.raises(ValueError):
        fa_literal(G, 5, 0.0, 1, 0.0)
    with pytest.raises(ValueError):
        fa_literal(G, 2, -1.0, 1, 0.0)
    with pytest.raises(ValueError):
        fa_literal(G, 2, 0.0, 0, 0.0)
