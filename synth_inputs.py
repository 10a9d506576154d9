"""Seeded synthetic gradient sets shaped like the Flag Aggregator paper's workloads.

This module only draws random numbers and lays them out in memory.  It holds
none of the aggregator's arithmetic, so both the CPU oracle's tests and the HIP
path's tests/bench may import it without sharing any method code.

Layout returned everywhere: *worker-major* -- a C-contiguous array ``Gw`` of
shape ``[p, n]`` whose row ``i`` is worker ``i``'s flat gradient ``g_i``.  The
paper's gradient matrix (Sec. 2.1, ``G`` with the ``g_i`` as columns) is
``Gw.T``.

The datasets, models and real gradients of the paper's experiments
(Sec. 3 "Setup": ResNet-18 / CIFAR-10, ResNet-50 / Tiny ImageNet, small CNN /
MNIST with up to 60 workers) are not available; only their shapes (p, n), the
Byzantine fractions and the attack styles (random gradients, sign flip with
amplification, colluding workers) are taken.

Draw order is fixed (and part of the recipe): ``mu`` (and any other shared
vectors) first, then the Byzantine index set, then the worker columns
``i = 0..p-1`` in order.  Every column is generated in fp64 and rounded once to
the storage dtype; the rounded array is what every consumer sees.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class Workload:
    """One aggregation problem: shape, solver arguments and the input recipe."""
    name: str
    p: int            # number of workers (columns of G)
    n: int            # gradient length (rows of G)
    m: int            # subspace dimension
    lam: float        # regularisation weight lambda of Eq. 5
    iters: int        # IRLS solves
    f: int            # number of Byzantine workers
    dtype: str        # storage: "f32" or "bf16"
    recipe: str       # which generator below

    def with_n(self, n: int) -> "Workload":
        return replace(self, n=int(n), name=f"{self.name}@n={int(n)}")

    def with_lam(self, lam: float) -> "Workload":
        return replace(self, lam=float(lam))


# The five configurations (cfg1..cfg5).  cfg2 is the one the headline metric is
# quoted on.
WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", p=7, n=100_000, m=4, lam=1.0, iters=10, f=1,
                     dtype="f32", recipe="signflip10"),
    "cfg2": Workload("cfg2", p=15, n=11_200_000, m=8, lam=1.0, iters=20, f=3,
                     dtype="f32", recipe="mixed_attack"),
    "cfg3": Workload("cfg3", p=15, n=25_600_000, m=8, lam=1.0, iters=20, f=3,
                     dtype="f32", recipe="student_collude"),
    "cfg4": Workload("cfg4", p=32, n=124_000_000, m=16, lam=1.0, iters=15, f=6,
                     dtype="bf16", recipe="lowrank_noise"),
    "cfg5": Workload("cfg5", p=64, n=50_000_000, m=32, lam=1.0, iters=30, f=12,
                     dtype="f32", recipe="two_cluster"),
}


def f32_to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """Round fp32 values to bfloat16 (round-to-nearest-even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def _store(col64: np.ndarray, dtype: str) -> np.ndarray:
    c32 = col64.astype(np.float32)
    if dtype == "f32":
        return c32
    if dtype == "bf16":
        return f32_to_bf16_bits(c32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


def _rms(x: np.ndarray) -> float:
    return float(np.sqrt(np.mean(x * x)))


def make_inputs(w: Workload, seed: int) -> Tuple[np.ndarray, dict]:
    """Return ``(Gw, meta)`` for workload ``w`` and ``seed``.

    ``Gw`` is ``[p, n]`` float32 (or uint16 bf16 bit patterns when
    ``w.dtype == "bf16"``).  ``meta`` records the Byzantine indices.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    p, n, f = w.p, w.n, w.f
    out = np.empty((p, n), dtype=np.float32 if w.dtype == "f32" else np.uint16)
    meta: dict = {"seed": seed, "recipe": w.recipe}

    if w.recipe == "signflip10":
        # honest: mu + 0.1 N(0, I), mu ~ N(0, I_n); Byzantine: 10x amplified sign flip.
        mu = rng.standard_normal(n)
        byz = np.sort(rng.choice(p, f, replace=False))
        for i in range(p):
            if i in byz:
                col = -10.0 * mu
            else:
                col = mu + 0.1 * rng.standard_normal(n)
            out[i] = _store(col, w.dtype)

    elif w.recipe == "mixed_attack":
        # honest: mu + sigma N(0, I), sigma = 0.5 rms(mu).  Each Byzantine column is
        # one of {N(0, 100 sigma^2 I), -4 mu, 1000 * random unit vector}, chosen uniformly.
        mu = rng.standard_normal(n)
        sigma = 0.5 * _rms(mu)
        byz = np.sort(rng.choice(p, f, replace=False))
        kinds = []
        for i in range(p):
            if i in byz:
                kind = int(rng.integers(0, 3))
                kinds.append(kind)
                if kind == 0:
                    col = 10.0 * sigma * rng.standard_normal(n)
                elif kind == 1:
                    col = -4.0 * mu
                else:
                    u = rng.standard_normal(n)
                    col = u * (1000.0 / np.sqrt(np.dot(u, u)))
            else:
                col = mu + sigma * rng.standard_normal(n)
            out[i] = _store(col, w.dtype)
        meta["byz_kinds"] = kinds

    elif w.recipe == "student_collude":
        # honest: mu + sigma * t_3 per coordinate, sigma = 0.5 rms(mu).
        # Byzantine (colluding): -mu + N(0, 0.01) jitter, 0.01 read as the variance.
        mu = rng.standard_normal(n)
        sigma = 0.5 * _rms(mu)
        byz = np.sort(rng.choice(p, f, replace=False))
        for i in range(p):
            if i in byz:
                col = -mu + 0.1 * rng.standard_normal(n)
            else:
                col = mu + sigma * rng.standard_t(3.0, n)
            out[i] = _store(col, w.dtype)

    elif w.recipe == "lowrank_noise":
        # honest: mu + U z_i + noise, U in R^{n x 4} Gaussian, z_i ~ N(0, I_4),
        # noise sigma = 0.5 rms(mu) (scale fixed here).  Byzantine: N(0, 100 sigma^2 I).
        mu = rng.standard_normal(n)
        U = [rng.standard_normal(n) for _ in range(4)]
        sigma = 0.5 * _rms(mu)
        byz = np.sort(rng.choice(p, f, replace=False))
        for i in range(p):
            if i in byz:
                col = 10.0 * sigma * rng.standard_normal(n)
            else:
                z = rng.standard_normal(4)
                col = mu + sigma * rng.standard_normal(n)
                for k in range(4):
                    col += z[k] * U[k]
            out[i] = _store(col, w.dtype)

    elif w.recipe == "two_cluster":
        # honest: 70/30 mixture of two centres mu_1, mu_2 plus N(0, sigma^2),
        # sigma = 0.5 rms(mu_1) (scale fixed here).  Byzantine: alternately -4 mu_1
        # (sign flip) and N(0, 100 sigma^2 I) (large-norm noise).
        mu1 = rng.standard_normal(n)
        mu2 = rng.standard_normal(n)
        sigma = 0.5 * _rms(mu1)
        byz = np.sort(rng.choice(p, f, replace=False))
        nb = 0
        for i in range(p):
            if i in byz:
                if nb % 2 == 0:
                    col = -4.0 * mu1
                else:
                    col = 10.0 * sigma * rng.standard_normal(n)
                nb += 1
            else:
                centre = mu1 if rng.random() < 0.7 else mu2
                col = centre + sigma * rng.standard_normal(n)
            out[i] = _store(col, w.dtype)
    else:
        raise ValueError(f"unknown recipe {w.recipe!r}")

    meta["byzantine"] = [int(b) for b in byz]
    return out, meta


# ---------------------------------------------------------------------------------------------
# The two widest configurations at their full size: 4.6e9 and 3.3e9 normal deviates.  One
# sequential stream takes minutes there, so the same recipes are drawn chunk by chunk from
# independent seeded streams, one per (vector, chunk of rows), on several threads.  The numbers
# differ from make_inputs' (another stream layout), the distributions, scales and structure do
# not; the result depends on (workload, seed, chunk_rows) only, not on the thread count.
CHUNK_ROWS = 1 << 22

_VEC_MU, _VEC_MU2, _VEC_U0, _VEC_COL0 = 0, 1, 2, 16   # stream ids of the vectors of a recipe


def _chunk_normal(seed: int, vec: int, chunk: int, rows: int) -> np.ndarray:
    ss = np.random.SeedSequence([int(seed), int(vec), int(chunk), 0x5EED])
    return np.random.Generator(np.random.PCG64(ss)).standard_normal(rows)


def make_inputs_chunked(w: Workload, seed: int, threads: int = 16,
                        chunk_rows: int = CHUNK_ROWS) -> Tuple[np.ndarray, dict]:
    """``(Gw, meta)`` like ``make_inputs`` for the recipes of the two widest configurations
    (``lowrank_noise``, ``two_cluster``), drawn in parallel (see above)."""
    from concurrent.futures import ThreadPoolExecutor
    if w.recipe not in ("lowrank_noise", "two_cluster"):
        raise ValueError(f"no chunked generator for recipe {w.recipe!r}")
    p, n, f = w.p, w.n, w.f
    small = np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), 0xB12])))
    byz = np.sort(small.choice(p, f, replace=False))
    z = small.standard_normal((p, 4))            # lowrank_noise: coordinates in span(U)
    in_first = small.random(p) < 0.7             # two_cluster: which centre a worker follows
    chunks = [(c, a, min(n, a + chunk_rows)) for c, a in enumerate(range(0, n, chunk_rows))]
    out = np.empty((p, n), dtype=np.float32 if w.dtype == "f32" else np.uint16)

    def mu_square_sum(ch):
        c, a, b = ch
        x = _chunk_normal(seed, _VEC_MU, c, b - a)
        return float(np.dot(x, x))

    def fill(ch):
        c, a, b = ch
        rows = b - a
        mu = _chunk_normal(seed, _VEC_MU, c, rows)
        if w.recipe == "lowrank_noise":
            U = [_chunk_normal(seed, _VEC_U0 + k, c, rows) for k in range(4)]
        else:
            mu2 = _chunk_normal(seed, _VEC_MU2, c, rows)
        nb = 0
        for i in range(p):
            if w.recipe == "lowrank_noise":
                if i in byz:
                    col = 10.0 * sigma * _chunk_normal(seed, _VEC_COL0 + i, c, rows)
                else:
                    col = mu + sigma * _chunk_normal(seed, _VEC_COL0 + i, c, rows)
                    for k in range(4):
                        col += z[i, k] * U[k]
            else:
                if i in byz:
                    if nb % 2 == 0:
                        col = -4.0 * mu
                    else:
                        col = 10.0 * sigma * _chunk_normal(seed, _VEC_COL0 + i, c, rows)
                    nb += 1
                else:
                    col = (mu if in_first[i] else mu2) + sigma * _chunk_normal(
                        seed, _VEC_COL0 + i, c, rows)
            out[i, a:b] = _store(col, w.dtype)
        return rows

    with ThreadPoolExecutor(max_workers=max(1, int(threads))) as pool:
        # sigma = 0.5 rms(mu), added up chunk by chunk in chunk order
        sigma = 0.5 * float(np.sqrt(sum(pool.map(mu_square_sum, chunks)) / n))
        done = sum(pool.map(fill, chunks))
    assert done == n
    return out, {"seed": seed, "recipe": w.recipe, "byzantine": [int(b) for b in byz],
                 "generator": "chunked"}


def random_dense(p: int, n: int, seed: int, scale: float = 1.0) -> np.ndarray:
    """Plain i.i.d. N(0, scale^2) worker-major fp32 matrix (unit tests of single kernels)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return (scale * rng.standard_normal((p, n))).astype(np.float32)
