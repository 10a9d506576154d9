"""CPU oracle for the Flag Aggregator (FA) aggregation step.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 NumPy.  Only the tests, the smoke check and the bench's
``cpu_baseline`` leg may import this package; the product path (the HIP library
and its Python binding) never does, and this file shares no code with it.

What it computes (paper: "Flag Aggregator", Almasi et al., arXiv 2302.05865)
---------------------------------------------------------------------------
Given the gradient matrix ``G in R^{n x p}`` (column ``i`` = worker gradient
``g_i``, Sec. 2.1), find an orthonormal ``Y in R^{n x m}`` for the FA objective
(Eq. 5 with the data-dependent regulariser, option (2) of Sec. 2.3)

    A(Y) = sum_i sqrt(1 - ||Y^T g_i||^2 / ||g_i||^2)
         + lam/(p-1) * sum_{i != j} sqrt(1 - ||Y^T (g_i-g_j)||^2 / D_ij^2),
    D_ij^2 = ||g_i - g_j||^2,

by iteratively re-weighted least squares, i.e. by repeatedly solving weighted
PCA problems ("IRLS"/"flag mean", Alg. 1 step "IRLS", Sec. 3 "Implementation
Details", Appendix E.2 on PCA), and return the update direction
``d = (1/p) Y Y^T G 1`` (Alg. 1, "Obtain gradient direction").

Readings of the paper taken here (the paper names the IRLS but does not print it)
--------------------------------------------------------------------------------
* Update = majorise-minimise step for the concave square root:
  ``sqrt(x) <= sqrt(x0) + (x-x0)/(2 sqrt(x0))``.  With residuals
  ``rho = 1 - (explained variance)`` the next ``Y`` maximises
  ``sum_i w_i v_i + lam/(p-1) sum_{i!=j} w_ij u_ij`` with ``w = rho^{-1/2}``,
  i.e. ``Y`` = the ``m`` leading left singular vectors of the matrix whose
  columns are ``sqrt(w_i) g_i/||g_i||`` and
  ``sqrt(lam/(p-1)) sqrt(w_ij) (g_i-g_j)/D_ij`` (all ordered pairs i != j).
* Start from uniform weights, so the first solve is PCA of the normalised
  gradients (Appendix E.2: one FA iteration with uniform weights is PCA).
* ``iters`` counts solves including that first one.
* The pair sum runs over ordered pairs as printed (each unordered pair twice).
* ``D_ij`` uses the raw gradients as printed; the output uses the raw ``G``.
* A zero-norm column, or a pair with ``D_ij = 0``, has its term dropped
  (weight 0, no contribution to the objective); the column still counts in 1/p.
  "``D_ij = 0``" is read as ``D_ij^2 <= tau_pair (||g_i||^2 + ||g_j||^2)`` with
  ``tau_pair = 1e-12``: two gradients closer than 1e-6 of their size are duplicates
  (exact duplicates give exactly 0 in the literal form; the floor keeps the
  ``R``-factor form, whose differences carry rounding noise, on the same branch).
* Weight floor: ``w = max(rho, delta)^{-1/2}`` with ``delta = 1e-6`` (the
  convergence proof in Appendix D perturbs the square root's argument by a
  positive constant for the same reason).
* Stop test: ``|A_{k-1} - A_k| < tol`` on the (unclamped) objective; ``tol = 0``
  never stops early.  No revert if the objective rises.

"parity unpinned": the weight floor ``delta``, the stop rule and the ordered
pair factor are readings, not values fixed by the paper; the tests pin the
ordered-pair factor and the weight exponent through stationarity of Eq. 5, but
``delta`` and the stop rule are pinned only by being stated here.
"""
from __future__ import annotations

from typing import Dict, Iterator, List, Optional, Tuple

import numpy as np

DELTA_DEFAULT = 1e-6
TAU_PAIR_DEFAULT = 1e-12


def decode_bf16(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 values (exact)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32)


def as_f64_matrix(Gw: np.ndarray) -> np.ndarray:
    """Worker-major storage ``[p, n]`` (fp32, fp64 or bf16 bits) -> math ``G`` (n x p) fp64."""
    if Gw.dtype == np.uint16:
        Gw = decode_bf16(Gw)
    return np.asarray(Gw, dtype=np.float64).T


def fa_literal(G: np.ndarray, m: int, lam: float, iters: int, tol: float,
               delta: float = DELTA_DEFAULT,
               tau_pair: float = TAU_PAIR_DEFAULT, a: float = 2.0) -> Dict[str, object]:
    """FA by IRLS, taken literally on the n x p matrix ``G`` (use for small n).

    Follows Eq. 5 / Sec. 2.3 option (2) for the objective, Alg. 1 for the output.
    ``a`` is the constant of the Taylor step in Sec. 2.2 ("Step 2"): every term of the
    objective is ``(1 - v)^(1/a)``; FA proper is ``a = 2`` (the square roots of Eq. 5).
    The IRLS weight of a term is the slope of ``rho^(1/a)`` at the current residual,
    ``max(rho, delta)^(1/a - 1)`` up to the common factor ``1/a``.
    Returns a dict with ``out`` (n), ``Y`` (n x m), ``v`` (p), ``w`` (p),
    ``u``/``w_pair`` (p x p, zero diagonal), ``objective`` (list), ``iters_done``.
    """
    G = np.asarray(G, dtype=np.float64)
    n, p = G.shape
    if not (1 <= m <= p):
        raise ValueError("need 1 <= m <= p")
    if n < m:
        raise ValueError("need n >= m")
    if iters < 1 or lam < 0 or tol < 0 or not (a >= 1.0):
        raise ValueError("bad solver arguments")

    # Explained-variance denominators ||g_i||^2 (Sec. 2.1) and normalised gradients
    # g_i/||g_i|| (Appendix B, the m = 1 reformulation; Appendix D on normalising).
    s = np.array([G[:, i] @ G[:, i] for i in range(p)])
    live = s > 0
    Gn = np.zeros_like(G)
    for i in range(p):
        if live[i]:
            Gn[:, i] = G[:, i] / np.sqrt(s[i])

    # Pairwise differences and D_ij^2 = ||g_i - g_j||^2 (Sec. 2.3 option (2)), ordered pairs.
    use_pairs = lam > 0 and p > 1
    pairs: List[Tuple[int, int]] = []
    if use_pairs:
        pairs = [(i, j) for i in range(p) for j in range(p) if i != j]
    q = len(pairs)
    Dn = np.zeros((n, q))
    D2 = np.zeros(q)
    live_pair = np.zeros(q, dtype=bool)
    for k, (i, j) in enumerate(pairs):
        d = G[:, i] - G[:, j]
        D2[k] = d @ d
        live_pair[k] = D2[k] > tau_pair * (s[i] + s[j])
        if live_pair[k]:
            Dn[:, k] = d / np.sqrt(D2[k])
    coef = lam / (p - 1) if use_pairs else 0.0

    w = live.astype(np.float64)            # uniform start
    wp = live_pair.astype(np.float64)
    objective: List[float] = []
    Y = None
    v = u = None
    for k in range(iters):
        # weighted PCA: m leading left singular vectors of the re-weighted columns
        X = np.concatenate([Gn * np.sqrt(w)[None, :],
                            np.sqrt(coef) * Dn * np.sqrt(wp)[None, :]], axis=1)
        U, _, _ = np.linalg.svd(X, full_matrices=False)   # singular values descending
        Y = U[:, :m]
        # explained variances (Sec. 2.1 "value" of a worker; pair analogue in Sec. 2.3)
        v = np.sum((Y.T @ Gn) ** 2, axis=0)
        u = np.sum((Y.T @ Dn) ** 2, axis=0)
        rho = np.maximum(1.0 - v, 0.0)
        rho_p = np.maximum(1.0 - u, 0.0)
        obj = float(np.sum((rho ** (1.0 / a))[live]) + coef * np.sum((rho_p ** (1.0 / a))[live_pair]))
        objective.append(obj)
        if k > 0 and abs(objective[-2] - obj) < tol:
            break
        w = np.where(live, np.maximum(rho, delta) ** (1.0 / a - 1.0), 0.0)
        wp = np.where(live_pair, np.maximum(rho_p, delta) ** (1.0 / a - 1.0), 0.0)

    # d = (1/p) Y Y^T G 1 with the raw G (Alg. 1)
    out = Y @ (Y.T @ G.sum(axis=1)) / p

    u_mat = np.zeros((p, p))
    wp_mat = np.zeros((p, p))
    for k, (i, j) in enumerate(pairs):
        u_mat[i, j] = u[k]
        wp_mat[i, j] = wp[k]
    return {"out": out, "Y": Y, "v": np.where(live, v, 0.0), "w": w, "u": u_mat,
            "w_pair": wp_mat, "objective": objective, "iters_done": len(objective),
            "s": s}


def _row_chunks(n: int, chunk_rows: int) -> Iterator[Tuple[int, int]]:
    a = 0
    while a < n:
        b = min(n, a + chunk_rows)
        yield a, b
        a = b


def tsqr_r(Gw: np.ndarray, chunk_rows: int = 1 << 20) -> np.ndarray:
    """Upper-triangular ``R`` (p x p) of ``G = Q R`` by a chunked tall-skinny QR in fp64.

    ``Gw`` is worker-major storage ``[p, n]``.  ``R^T R = G^T G`` (an isometry of the
    columns), which is all FA needs from the n-sized data besides the final product.
    """
    p, n = Gw.shape
    if n < p:
        # pad with zero rows so every block has at least p rows
        G = np.zeros((p, p))
        G[:n] = as_f64_matrix(Gw)
        return np.linalg.qr(G, mode="r")
    blocks = []
    for a, b in _row_chunks(n, chunk_rows):
        blk = as_f64_matrix(Gw[:, a:b])
        if blk.shape[0] < p:
            pad = np.zeros((p, p))
            pad[:blk.shape[0]] = blk
            blk = pad
        blocks.append(np.linalg.qr(blk, mode="r"))
    if len(blocks) == 1:
        return blocks[0]
    return np.linalg.qr(np.vstack(blocks), mode="r")


def fa_scaled(Gw: np.ndarray, m: int, lam: float, iters: int, tol: float,
              delta: float = DELTA_DEFAULT, tau_pair: float = TAU_PAIR_DEFAULT,
              chunk_rows: int = 1 << 20, a: float = 2.0) -> Dict[str, object]:
    """FA for large n: the literal IRLS run on the ``R`` factor of ``G = Q R``.

    ``Q`` has orthonormal columns, so norms, pairwise distances and explained
    variances of the ``g_i`` equal those of the columns of ``R``; the subspace is
    ``Y = Q U`` with ``U`` the literal solution for ``R``, and
    ``d = (1/p) Y Y^T G 1 = Q t``, ``t = (1/p) U U^T R 1``.  Because ``t`` lies in
    range(R), ``d = G c`` with ``c`` the minimum-norm solution of ``R c = t``.

    ``Gw`` is worker-major storage ``[p, n]`` (fp32 or bf16 bits).  Returns the
    literal result's fields for ``R`` plus ``out`` (n, fp64), ``c`` (p), ``A``
    (p x m with ``Y = G A``), ``K`` (= R^T R = G^T G) and ``R``.
    """
    p, n = Gw.shape
    R = tsqr_r(Gw, chunk_rows)
    res = fa_literal(R, m, lam, iters, tol, delta, tau_pair, a)
    U = res["Y"]                                   # p x m, orthonormal
    t = U @ (U.T @ R.sum(axis=1)) / p
    c = np.linalg.lstsq(R, t, rcond=None)[0]
    A = np.linalg.lstsq(R, U, rcond=None)[0]
    out = np.empty(n)
    for a, b in _row_chunks(n, chunk_rows):
        out[a:b] = as_f64_matrix(Gw[:, a:b]) @ c
    res = dict(res)
    res.update({"out": out, "c": c, "A": A, "R": R, "K": R.T @ R, "U": U})
    del res["Y"]
    return res


def projector_difference(A1: np.ndarray, A2: np.ndarray, R: np.ndarray) -> float:
    """Frobenius norm of ``P1 - P2`` for ``P_k = (G A_k)(G A_k)^T``, given any factor ``R``
    with ``G = Q R`` (``Q`` with orthonormal columns; e.g. the ``R`` of ``fa_scaled``).

    ``P_k = Q (R A_k)(R A_k)^T Q^T``, hence
    ``||P1 - P2||_F = ||(R A1)(R A1)^T - (R A2)(R A2)^T||_F``.
    Components of ``A_k`` in the null space of ``G`` (free when the gradients are linearly
    dependent) are annihilated by ``R`` itself, to rounding, before anything is subtracted.
    (Forms that go through ``K = G^T G`` -- ``sqrt(tr((M K)^2))`` or ``K^{1/2}`` -- see
    the null space only to ``sqrt(eps)`` and have a noise floor near 1e-8 there.)
    """
    W1, W2 = R @ A1, R @ A2
    return float(np.linalg.norm(W1 @ W1.T - W2 @ W2.T))


def basis_products(G: np.ndarray, Y: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """``(Y^T Y, Y^T G)`` for ``G`` (n x p) and ``Y`` (n x m), written out as the definition
    (Sec. 2.1: ``Y`` has orthonormal columns, so the first is the identity for a valid basis;
    the explained variance of worker ``i`` is ``sum_a (Y^T G)[a, i]^2 / ||g_i||^2``)."""
    G = np.asarray(G, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    return Y.T @ Y, Y.T @ G


def fa_literal_grouped(G: np.ndarray, sizes: List[int], m: int, lam: float, iters: int,
                       tol: float, delta: float = DELTA_DEFAULT,
                       tau_pair: float = TAU_PAIR_DEFAULT, a: float = 2.0) -> Dict[str, object]:
    """FA when worker ``i`` sends ``k_i = sizes[i]`` gradients: ``g_i`` is the n x k_i block of
    consecutive columns of ``G`` (Sec. 2.1; Sec. 2.2, the extension to ``g_i in R^{n x k}``;
    Appendix D works with such lists).

    The value of worker ``i`` is ``v_i = tr(g_i^T Y Y^T g_i) / tr(g_i^T g_i)``; every other
    step is ``fa_literal``'s with blocks in place of columns.  Readings (the paper does not
    spell these out): the pairwise term of Sec. 2.3 needs ``g_i - g_j`` and so exists only
    between workers with equal ``k``; its distance is the Frobenius one; the factor is
    ``lam / (P - 1)`` with ``P`` workers; a worker counts once in the output whatever its
    ``k``: ``d = (1/P) Y Y^T sum_i mean_columns(g_i)``.
    Returns ``out``, ``Y``, ``v`` and ``w`` (per worker), ``objective``, ``iters_done``.
    """
    G = np.asarray(G, dtype=np.float64)
    n, q = G.shape
    P = len(sizes)
    if P < 1 or any(k < 1 for k in sizes) or sum(sizes) != q:
        raise ValueError("sizes must be positive and add up to the number of columns")
    if not (1 <= m <= q) or n < m:
        raise ValueError("need 1 <= m <= number of columns <= ... and n >= m")
    if iters < 1 or lam < 0 or tol < 0 or not (a >= 1.0):
        raise ValueError("bad solver arguments")
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(int)
    blocks = [G[:, off[i]:off[i + 1]] for i in range(P)]
    s = np.array([np.sum(b * b) for b in blocks])                 # tr(g_i^T g_i)
    live = s > 0
    Gn = [b / np.sqrt(s[i]) if live[i] else np.zeros_like(b) for i, b in enumerate(blocks)]

    use_pairs = lam > 0 and P > 1
    coef = lam / (P - 1) if use_pairs else 0.0
    Dn: List[np.ndarray] = []
    if use_pairs:
        for i in range(P):
            for j in range(P):
                if i == j or sizes[i] != sizes[j]:
                    continue
                d = blocks[i] - blocks[j]
                d2 = np.sum(d * d)
                if d2 > tau_pair * (s[i] + s[j]):
                    Dn.append(d / np.sqrt(d2))

    w = live.astype(np.float64)
    wp = np.ones(len(Dn))
    objective: List[float] = []
    Y = None
    v = np.zeros(P)
    for k in range(iters):
        cols = [np.sqrt(w[i]) * Gn[i] for i in range(P)]
        cols += [np.sqrt(coef * wp[t]) * Dn[t] for t in range(len(Dn))]
        U, _, _ = np.linalg.svd(np.concatenate(cols, axis=1), full_matrices=False)
        Y = U[:, :m]
        v = np.array([np.sum((Y.T @ Gn[i]) ** 2) for i in range(P)])
        u = np.array([np.sum((Y.T @ d) ** 2) for d in Dn])
        rho = np.maximum(1.0 - v, 0.0)
        rho_p = np.maximum(1.0 - u, 0.0)
        obj = float(np.sum((rho ** (1.0 / a))[live]) + coef * np.sum(rho_p ** (1.0 / a)))
        objective.append(obj)
        if k > 0 and abs(objective[-2] - obj) < tol:
            break
        w = np.where(live, np.maximum(rho, delta) ** (1.0 / a - 1.0), 0.0)
        wp = np.maximum(rho_p, delta) ** (1.0 / a - 1.0)

    gbar = sum(b.mean(axis=1) for b in blocks)
    out = Y @ (Y.T @ gbar) / P
    return {"out": out, "Y": Y, "v": np.where(live, v, 0.0), "w": w, "objective": objective,
            "iters_done": len(objective), "s": s}


def multi_krum(G: np.ndarray, f: int, q: int) -> Dict[str, object]:
    """Multi-Krum, the distance-based aggregator the paper compares with most (Sec. 3
    "Baselines"; Sec. 2.3 on aggregators "that benefit from pairwise distances"; Appendix E):
    the paper only cites it, so this restates the published rule (Blanchard et al., 2017) on the
    columns of ``G`` (n x p).  Worker ``i`` is scored by the sum of its squared distances to its
    ``p - f - 2`` nearest other workers (``f`` = number of Byzantine workers provided for); the
    ``q`` workers with the smallest scores are averaged.  Ties (equal scores, equal distances)
    go to the smaller index.  Returns ``out`` (n), ``scores`` (p), ``selected`` (p, 0/1)."""
    G = np.asarray(G, dtype=np.float64)
    n, p = G.shape
    k = p - f - 2
    if f < 0 or k < 1 or not (1 <= q <= p):
        raise ValueError("need f >= 0, p - f - 2 >= 1 and 1 <= q <= p")
    scores = np.zeros(p)
    for i in range(p):
        d = sorted(float(np.sum((G[:, i] - G[:, j]) ** 2)) for j in range(p) if j != i)
        acc = 0.0
        for x in d[:k]:                      # ascending order, the order the library adds in
            acc += x
        scores[i] = acc
    order = sorted(range(p), key=lambda i: (scores[i], i))
    selected = np.zeros(p, dtype=np.int32)
    selected[order[:q]] = 1
    out = G[:, selected == 1].sum(axis=1) / q
    return {"out": out, "scores": scores, "selected": selected}
