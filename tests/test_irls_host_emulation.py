"""Host logic of the library's p x p solver (csrc/fa_irls_core.inc) against the oracle.

The solver text is written as barrier-separated parallel-for phases; tests/emul builds it as
a sequential host program (test-only, never part of libfa.so).  Comparing that build with the
oracle checks the solver's indexing, Jacobi ordering, rank handling and coefficient formulas
here, without a GPU.  The GPU tests run the same text as a kernel.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import synth_inputs as si
from oracle import (as_f64_matrix, fa_literal, fa_literal_grouped, fa_scaled,
                    projector_difference)
from paper_2302_05865_amd._ctypes_defs import FaInfo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def emul(tmp_path_factory):
    out = tmp_path_factory.mktemp("emul") / "libirls_emul.so"
    subprocess.check_call(["g++", "-O2", "-shared", "-fPIC", "-I", os.path.join(ROOT, "include"),
                           "-I", os.path.join(ROOT, "paper_2302_05865_amd", "csrc"),
                           os.path.join(ROOT, "tests", "emul", "irls_emul.cpp"), "-o", str(out)])
    lib = ctypes.CDLL(str(out))

    def run(K, m, lam, iters, tol, delta=1e-6, rank_tol=1e-12, pair_tol=1e-12, stepwise=False,
            a=None, sizes=None):
        K = np.ascontiguousarray(K, dtype=np.float64)
        p = K.shape[0]
        info = FaInfo()
        c = np.zeros(p)
        d = ctypes.c_double
        if sizes is not None:
            sz = (ctypes.c_int * len(sizes))(*sizes)
            rc = lib.fa_irls_emulate_grouped(
                K.ctypes.data_as(ctypes.c_void_p), p, sz, len(sizes), m, d(lam), iters, d(tol),
                d(delta), d(rank_tol), d(pair_tol), c.ctypes.data_as(ctypes.c_void_p),
                ctypes.byref(info))
            assert rc == 0
            return c, info
        if a is not None:
            rc = lib.fa_irls_emulate_exponent(
                K.ctypes.data_as(ctypes.c_void_p), p, m, d(lam), iters, d(tol), d(delta),
                d(rank_tol), d(pair_tol), d(a), c.ctypes.data_as(ctypes.c_void_p),
                ctypes.byref(info))
            assert rc == 0
            return c, info
        fn = lib.fa_irls_emulate_stepwise if stepwise else lib.fa_irls_emulate
        rc = fn(K.ctypes.data_as(ctypes.c_void_p), p, m, d(lam), iters, d(tol),
                d(delta), d(rank_tol), d(pair_tol),
                c.ctypes.data_as(ctypes.c_void_p), ctypes.byref(info))
        assert rc == 0
        return c, info
    return run


@pytest.mark.parametrize("name,n", [("cfg1", 20000), ("cfg2", 50000), ("cfg3", 50000),
                                    ("cfg4", 30000), ("cfg5", 20000)])
@pytest.mark.parametrize("seed", [0, 1])
def test_solver_text_matches_oracle_on_workload_shapes(emul, name, n, seed):
    w = si.WORKLOADS[name].with_n(n)
    Gw, _ = si.make_inputs(w, seed)
    ref = fa_scaled(Gw, w.m, w.lam, w.iters, 0.0)
    G = as_f64_matrix(Gw)
    K = G.T @ G
    c, info = emul(K, w.m, w.lam, w.iters, 0.0)
    out = G @ c
    assert info.status == 0 and info.iters_done == w.iters
    assert np.linalg.norm(out - ref["out"]) <= 1e-9 * np.linalg.norm(ref["out"])
    A = np.array(info.A[:w.p * w.m]).reshape(w.p, w.m)
    assert projector_difference(A, ref["A"], ref["R"]) <= 1e-9
    assert np.allclose(np.array(info.objective[:w.iters]), ref["objective"], atol=1e-6)
    assert np.allclose(np.array(info.v[:w.p]), ref["v"], atol=1e-9)


@pytest.mark.parametrize("lam", [0.0, 1.0])
def test_solver_text_small_cases(emul, lam):
    rng = np.random.default_rng(0)
    for (n, p, m) in [(40, 1, 1), (40, 2, 1), (40, 3, 3), (60, 9, 4), (50, 16, 8), (80, 17, 5)]:
        G = rng.standard_normal((n, p)) * rng.uniform(0.3, 3, p)[None, :]
        ref = fa_literal(G, m, lam, 6, 0.0)
        c, info = emul(G.T @ G, m, lam, 6, 0.0)
        assert np.linalg.norm(G @ c - ref["out"]) <= 1e-8 * np.linalg.norm(ref["out"])
        assert info.rank == p


def test_solver_text_degenerate_inputs(emul):
    rng = np.random.default_rng(1)
    g = rng.standard_normal(30)
    # identical gradients, rank 1
    G = np.repeat(g[:, None], 5, axis=1)
    c, info = emul(G.T @ G, 3, 1.0, 4, 0.0)
    assert info.rank == 1 and np.allclose(G @ c, g, atol=1e-12)
    # a zero column and a duplicate pair
    G = rng.standard_normal((30, 6))
    G[:, 2] = 0.0
    G[:, 4] = G[:, 1]
    ref = fa_literal(G, 2, 1.0, 5, 0.0)
    c, info = emul(G.T @ G, 2, 1.0, 5, 0.0)
    assert info.rank == 4
    assert np.linalg.norm(G @ c - ref["out"]) <= 1e-10 * np.linalg.norm(ref["out"])
    # all zero / non-finite
    c, info = emul(np.zeros((4, 4)), 2, 1.0, 3, 0.0)
    assert info.status == 5 and np.all(c == 0)
    K = np.eye(4); K[1, 2] = K[2, 1] = np.nan
    c, info = emul(K, 2, 1.0, 3, 0.0)
    assert info.status == 4 and np.all(np.isnan(c))


def test_solver_text_stop_rule(emul):
    rng = np.random.default_rng(3)
    G = rng.standard_normal((40, 7)) * rng.uniform(0.3, 3, 7)[None, :]
    full = fa_literal(G, 3, 1.0, 30, 0.0)
    early = fa_literal(G, 3, 1.0, 30, 1e-3)
    c, info = emul(G.T @ G, 3, 1.0, 30, 1e-3)
    assert info.iters_done == early["iters_done"] < 30
    assert np.linalg.norm(G @ c - early["out"]) <= 1e-10 * np.linalg.norm(early["out"])
    assert np.allclose(np.array(info.w[:7]), early["w"], rtol=1e-8)
    c, info = emul(G.T @ G, 3, 1.0, 30, 0.0)
    assert np.allclose(np.array(info.w[:7]), full["w"], rtol=1e-6)


@pytest.mark.parametrize("name,n", [("cfg1", 20000), ("cfg2", 50000), ("cfg5", 20000)])
def test_one_solve_per_call_through_the_resume_state_equals_one_call(emul, name, n):
    """The re-streaming schedule drives the IRLS one solve per launch; the weights travel
    through the resume state.  Same iterates as the single call (the eigenbasis restarts, so
    equal to rounding, not bitwise)."""
    w = si.WORKLOADS[name].with_n(n)
    Gw, _ = si.make_inputs(w, 0)
    G = as_f64_matrix(Gw)
    K = G.T @ G
    c1, i1 = emul(K, w.m, w.lam, w.iters, 0.0)
    c2, i2 = emul(K, w.m, w.lam, w.iters, 0.0, stepwise=True)
    assert i2.iters_done == w.iters == i1.iters_done
    assert np.allclose(np.array(i2.objective[:w.iters]), np.array(i1.objective[:w.iters]),
                       rtol=0, atol=1e-10)
    assert np.linalg.norm(G @ (c1 - c2)) <= 1e-10 * np.linalg.norm(G @ c1)


@pytest.mark.parametrize("a", [1.0, 1.5, 3.0])
def test_general_exponent_in_the_solver_text(emul, a):
    """Sec. 2.2, Step 2: terms (1 - v)^(1/a) with a other than 2 (the any-p solver only)."""
    w = si.WORKLOADS["cfg2"].with_n(30000)
    Gw, _ = si.make_inputs(w, 1)
    ref = fa_scaled(Gw, w.m, w.lam, 12, 0.0, a=a)
    G = as_f64_matrix(Gw)
    c, info = emul(G.T @ G, w.m, w.lam, 12, 0.0, a=a)
    assert np.linalg.norm(G @ c - ref["out"]) <= 1e-8 * np.linalg.norm(ref["out"])
    assert np.allclose(np.array(info.objective[:12]), ref["objective"], atol=1e-6)


@pytest.mark.parametrize("sizes,m,lam", [([2, 3, 1, 2, 2, 1], 3, 1.0), ([4, 4, 4], 5, 1.0),
                                         ([1, 1, 1, 1, 1], 2, 1.0), ([3, 2, 3, 2, 3], 4, 0.0),
                                         ([7], 2, 1.0)])
def test_workers_with_several_gradients_in_the_solver_text(emul, sizes, m, lam):
    """Sec. 2.1 / Sec. 2.2 extension: blocks of columns as workers, value
    tr(g^T Y Y^T g) / tr(g^T g); the solver text against the block oracle."""
    rng = np.random.default_rng(sum(sizes))
    q, n = sum(sizes), 200
    G = rng.standard_normal((n, q)) * rng.uniform(0.3, 3.0, q)[None, :]
    G[:, 0] += 2.0 * G[:, -1]
    ref = fa_literal_grouped(G, sizes, m, lam, 9, 0.0)
    c, info = emul(G.T @ G, m, lam, 9, 0.0, sizes=sizes)
    assert info.status == 0 and info.iters_done == 9
    assert np.linalg.norm(G @ c - ref["out"]) <= 1e-8 * np.linalg.norm(ref["out"])
    assert np.allclose(np.array(info.objective[:9]), ref["objective"], atol=1e-8)
    first = np.concatenate([[0], np.cumsum(sizes)[:-1]])
    assert np.allclose(np.array(info.v[:q])[first], ref["v"], atol=1e-8)
    # every column of a block reports its worker's value
    assert np.allclose(np.repeat(np.array(info.v[:q])[first], sizes), np.array(info.v[:q]))


def test_a_zero_block_is_a_dropped_worker_in_the_solver_text(emul):
    rng = np.random.default_rng(3)
    sizes = [2, 2, 3]
    G = rng.standard_normal((60, 7))
    G[:, 2:4] = 0.0
    ref = fa_literal_grouped(G, sizes, 2, 1.0, 6, 0.0)
    c, info = emul(G.T @ G, 2, 1.0, 6, 0.0, sizes=sizes)
    assert np.linalg.norm(G @ c - ref["out"]) <= 1e-8 * np.linalg.norm(ref["out"])
    assert np.allclose(np.array(info.objective[:6]), ref["objective"], atol=1e-8)
