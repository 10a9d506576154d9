"""ctypes binding with the same names as the C ABI (include/fa.h).

No arithmetic of the method lives here: the class below validates tensor types, extracts
raw device pointers / the current stream and forwards to ``libfa.so``.  If the library is
missing the import of a symbol fails loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

from ._ctypes_defs import (FA_BF16, FA_F32, FA_ITERS_MAX, FA_OK, FA_P_MAX, FaConfig, FaInfo)

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libfa.so"
_lib: Optional[ctypes.CDLL] = None

# every symbol include/fa.h declares
EXPORTED_SYMBOLS = (
    "fa_default_config", "fa_create", "fa_destroy", "fa_set_stream", "fa_aggregate",
    "fa_get_info", "fa_gram", "fa_gram_async", "fa_irls", "fa_combine", "fa_basis", "fa_check_basis", "fa_aggregate_grouped", "fa_multikrum",
    "fa_set_profiling",
    "fa_get_timings", "fa_enqueue_kernel", "fa_aggregate_restream", "fa_get_restream_info",
    "fa_status_string", "fa_version", "fa_aggregate_static", "fa_gram_begin", "fa_gram_update", "fa_gram_update_rows",
    "fa_aggregate_arrived",
)


class FaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = load_library().fa_status_string(status).decode()
        super().__init__(f"{where}: {msg} (fa_status {status})")


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library() -> ctypes.CDLL:
    """Load the in-tree ``libfa.so``; raise if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} is missing: build it with `python -m paper_2302_05865_amd.build` "
            "(the HIP library is the only implementation; there is no fallback)")
    lib = ctypes.CDLL(path)
    vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
    lib.fa_default_config.argtypes = [ctypes.POINTER(FaConfig)]
    lib.fa_default_config.restype = None
    lib.fa_create.argtypes = [ctypes.POINTER(FaConfig), ctypes.POINTER(vp)]
    lib.fa_create.restype = i32
    lib.fa_destroy.argtypes = [vp]
    lib.fa_destroy.restype = None
    lib.fa_set_stream.argtypes = [vp, vp]
    lib.fa_set_stream.restype = i32
    lib.fa_aggregate.argtypes = [vp, vp, i64, i32, i64, i32, dbl, i32, dbl, vp]
    lib.fa_aggregate.restype = i32
    lib.fa_get_info.argtypes = [vp, ctypes.POINTER(FaInfo)]
    lib.fa_get_info.restype = i32
    lib.fa_gram.argtypes = [vp, vp, i64, i32, i64, vp]
    lib.fa_gram.restype = i32
    lib.fa_gram_async.argtypes = [vp, vp, i64, i32, i64]
    lib.fa_gram_async.restype = i32
    lib.fa_irls.argtypes = [vp, vp, i32, i32, dbl, i32, dbl]
    lib.fa_irls.restype = i32
    lib.fa_combine.argtypes = [vp, vp, i64, i32, i64, vp, vp]
    lib.fa_combine.restype = i32
    lib.fa_basis.argtypes = [vp, vp, i64, i32, i64, i32, vp, i64]
    lib.fa_basis.restype = i32
    lib.fa_check_basis.argtypes = [vp, vp, i64, i32, i64, vp, i64, i32, vp, vp]
    lib.fa_check_basis.restype = i32
    lib.fa_aggregate_grouped.argtypes = [vp, vp, i64, i32, i64, vp, i32, i32, dbl, i32, dbl, vp]
    lib.fa_aggregate_grouped.restype = i32
    lib.fa_multikrum.argtypes = [vp, vp, i64, i32, i64, i32, i32, vp, vp, vp]
    lib.fa_multikrum.restype = i32
    lib.fa_set_profiling.argtypes = [vp, i32]
    lib.fa_set_profiling.restype = i32
    lib.fa_get_timings.argtypes = [vp, ctypes.POINTER(ctypes.c_float * 4)]
    lib.fa_get_timings.restype = i32
    lib.fa_enqueue_kernel.argtypes = [vp, i32, vp, i64, i32, i64, i32, dbl, i32, dbl, vp]
    lib.fa_enqueue_kernel.restype = i32
    lib.fa_aggregate_restream.argtypes = [vp, vp, i64, i32, i64, i32, dbl, i32, vp]
    lib.fa_aggregate_restream.restype = i32
    lib.fa_get_restream_info.argtypes = [vp, vp, vp, vp]
    lib.fa_get_restream_info.restype = i32
    lib.fa_aggregate_static.argtypes = [vp, i64, i32, i64, i32, i32, dbl, i32, dbl, vp, vp]
    lib.fa_aggregate_static.restype = i32
    lib.fa_gram_begin.argtypes = [vp, i32, i64]
    lib.fa_gram_begin.restype = i32
    lib.fa_gram_update.argtypes = [vp, vp, i64, i32]
    lib.fa_gram_update.restype = i32
    lib.fa_gram_update_rows.argtypes = [vp, vp, i64, i32, i64, i64]
    lib.fa_gram_update_rows.restype = i32
    lib.fa_aggregate_arrived.argtypes = [vp, vp, i64, i32, dbl, i32, dbl, vp]
    lib.fa_aggregate_arrived.restype = i32
    lib.fa_status_string.argtypes = [i32]
    lib.fa_status_string.restype = ctypes.c_char_p
    lib.fa_version.argtypes = []
    lib.fa_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


@dataclass
class FaInfoResult:
    status: int
    p: int
    m: int
    rank: int
    iters_done: int
    sweeps: int
    eigengap: float
    objective: np.ndarray
    s: np.ndarray
    v: np.ndarray
    w: np.ndarray
    c: np.ndarray
    A: np.ndarray   # p x m, Y = G A
    K: np.ndarray   # p x p


def _check(status: int, where: str) -> None:
    if status != FA_OK:
        raise FaError(status, where)


def fa_aggregate_static(G, m: int, lam: float, iters: int, tol: float, out):
    """``fa_aggregate`` through the entry point that allocates nothing (no context; the
    library's fixed device-resident workspace).  ``G``: ``[p, n]`` float32 or bfloat16 device
    tensor with unit inner stride, ``out``: contiguous float32 device tensor of n elements,
    both the caller's.  Enqueued on torch's current stream of the current device."""
    import torch
    if not G.is_cuda or G.dim() != 2 or G.stride(1) != 1 or G.dtype not in (torch.float32,
                                                                             torch.bfloat16):
        raise TypeError("G must be a float32/bfloat16 device tensor with unit inner stride")
    p, n = G.shape
    if not out.is_cuda or out.dtype != torch.float32 or out.numel() != n or not out.is_contiguous():
        raise TypeError("out must be a contiguous float32 device tensor of n elements")
    ldg = G.stride(0) if p > 1 else n
    _check(load_library().fa_aggregate_static(
        ctypes.c_void_p(G.data_ptr()), int(ldg), int(p), int(n),
        FA_F32 if G.dtype == torch.float32 else FA_BF16, int(m), float(lam), int(iters),
        float(tol), ctypes.c_void_p(out.data_ptr()),
        ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)), "fa_aggregate_static")
    return out


class FlagAggregator:
    """One library context (``fa_ctx``): workspace for gradients up to ``[p_max, n_max]``.

    ``G`` arguments are CUDA/HIP ``torch`` tensors of shape ``[p, n]`` (worker-major: row i is
    gradient i), dtype float32 (or bfloat16 for a bf16 context), with a contiguous last
    dimension.  Work is enqueued on ``torch.cuda.current_stream()`` at call time.
    """

    def __init__(self, n_max: int, p_max: int = FA_P_MAX, dtype: str = "f32",
                 clamp_delta: float = 1e-6, rank_tol: float = 1e-12, pair_tol: float = 1e-12,
                 exponent_a: float = 2.0, layout: str = "worker_major", solver: str = "auto",
                 wide_spin_budget: Optional[int] = None, gram: str = "auto"):
        import torch  # device memory and streams only
        self._torch = torch
        self._lib = load_library()
        cfg = FaConfig()
        self._lib.fa_default_config(ctypes.byref(cfg))
        cfg.n_max = int(n_max)
        cfg.p_max = int(p_max)
        cfg.dtype = {"f32": FA_F32, "bf16": FA_BF16}[dtype]
        cfg.stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        cfg.clamp_delta = clamp_delta
        cfg.rank_tol = rank_tol
        cfg.pair_tol = pair_tol
        cfg.exponent_a = exponent_a
        cfg.layout = {"worker_major": 0, "row_major": 1}[layout]
        cfg.solver = {"auto": 0, "jacobi16": 1, "jacobi": 2}[solver]
        cfg.gram = {"auto": 0, "fp64": 1, "bf16": 2}[gram]
        if wide_spin_budget is not None:
            cfg.wide_spin_budget = int(wide_spin_budget)
        self.layout = layout
        self.dtype = dtype
        self._ctx = ctypes.c_void_p()
        _check(self._lib.fa_create(ctypes.byref(cfg), ctypes.byref(self._ctx)), "fa_create")

    # -- plumbing -------------------------------------------------------------------------
    def close(self) -> None:
        if getattr(self, "_ctx", None) is not None and self._ctx:
            self._lib.fa_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _matrix(self, G):
        torch = self._torch
        want = torch.float32 if self.dtype == "f32" else torch.bfloat16
        if not G.is_cuda or G.dim() != 2 or G.dtype != want or G.stride(1) != 1:
            raise TypeError(f"G must be a device tensor of {want} with unit inner stride")
        if self.layout == "row_major":       # [n, p]: coordinate k's p values are contiguous
            n, p = G.shape
            ldg = G.stride(0) if n > 1 else p
            return ctypes.c_void_p(G.data_ptr()), int(ldg), int(p), int(n)
        p, n = G.shape
        ldg = G.stride(0) if p > 1 else n
        return ctypes.c_void_p(G.data_ptr()), int(ldg), int(p), int(n)

    def _use_current_stream(self) -> None:
        s = self._torch.cuda.current_stream().cuda_stream
        _check(self._lib.fa_set_stream(self._ctx, ctypes.c_void_p(s)), "fa_set_stream")

    # -- the C ABI, same names ------------------------------------------------------------
    def fa_aggregate(self, G, m: int, lam: float, iters: int, tol: float, out=None):
        ptr, ldg, p, n = self._matrix(G)
        torch = self._torch
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=G.device)
        if not out.is_cuda or out.dtype != torch.float32 or out.numel() != n or not out.is_contiguous():
            raise TypeError("out must be a contiguous float32 device tensor of n elements")
        self._use_current_stream()
        _check(self._lib.fa_aggregate(self._ctx, ptr, ldg, p, n, int(m), float(lam), int(iters),
                                      float(tol), ctypes.c_void_p(out.data_ptr())), "fa_aggregate")
        return out

    def fa_aggregate_grouped(self, G, sizes, m: int, lam: float, iters: int, tol: float, out=None):
        """Workers that send several gradients: ``sizes[i]`` consecutive columns of G each."""
        ptr, ldg, q, n = self._matrix(G)
        torch = self._torch
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=G.device)
        sz = (ctypes.c_int * len(sizes))(*[int(k) for k in sizes])
        self._use_current_stream()
        _check(self._lib.fa_aggregate_grouped(self._ctx, ptr, ldg, q, n, sz, len(sizes), int(m),
                                              float(lam), int(iters), float(tol),
                                              ctypes.c_void_p(out.data_ptr())),
               "fa_aggregate_grouped")
        return out

    def fa_multikrum(self, G, f: int, q: int, out=None):
        """Multi-Krum: (out, scores, selected) with scores float64[p] and selected int32[p]."""
        ptr, ldg, p, n = self._matrix(G)
        torch = self._torch
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=G.device)
        scores = np.zeros(p, dtype=np.float64)
        selected = np.zeros(p, dtype=np.int32)
        self._use_current_stream()
        _check(self._lib.fa_multikrum(self._ctx, ptr, ldg, p, n, int(f), int(q),
                                      ctypes.c_void_p(out.data_ptr()),
                                      scores.ctypes.data_as(ctypes.c_void_p),
                                      selected.ctypes.data_as(ctypes.c_void_p)), "fa_multikrum")
        return out, scores, selected

    def fa_aggregate_restream(self, G, m: int, lam: float, iters: int, out=None):
        ptr, ldg, p, n = self._matrix(G)
        torch = self._torch
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=G.device)
        if not out.is_cuda or out.dtype != torch.float32 or out.numel() != n or not out.is_contiguous():
            raise TypeError("out must be a contiguous float32 device tensor of n elements")
        self._use_current_stream()
        _check(self._lib.fa_aggregate_restream(self._ctx, ptr, ldg, p, n, int(m), float(lam),
                                               int(iters), ctypes.c_void_p(out.data_ptr())),
               "fa_aggregate_restream")
        self._restream_p = p
        return out

    def fa_get_restream_info(self, timings: bool = False):
        """(ms[2] or None, v_streamed[p], objective_streamed[FA_ITERS_MAX])"""
        ms = (ctypes.c_float * 2)()
        v = np.zeros(64, dtype=np.float64)
        obj = np.zeros(256, dtype=np.float64)
        _check(self._lib.fa_get_restream_info(
            self._ctx, ctypes.cast(ms, ctypes.c_void_p) if timings else None,
            v.ctypes.data_as(ctypes.c_void_p), obj.ctypes.data_as(ctypes.c_void_p)),
            "fa_get_restream_info")
        return (np.array(ms[:]) if timings else None), v[:getattr(self, "_restream_p", 64)], obj

    def fa_get_info(self) -> FaInfoResult:
        info = FaInfo()
        _check(self._lib.fa_get_info(self._ctx, ctypes.byref(info)), "fa_get_info")
        p, m = info.p, info.m
        it = info.iters_done
        return FaInfoResult(
            status=info.status, p=p, m=m, rank=info.rank, iters_done=it, sweeps=info.sweeps,
            eigengap=info.eigengap,
            objective=np.array(info.objective[:it], dtype=np.float64),
            s=np.array(info.s[:p]), v=np.array(info.v[:p]), w=np.array(info.w[:p]),
            c=np.array(info.c[:p]),
            A=np.array(info.A[:p * m], dtype=np.float64).reshape(p, m),
            K=np.array(info.K[:p * p], dtype=np.float64).reshape(p, p))

    def fa_gram(self, G) -> np.ndarray:
        ptr, ldg, p, n = self._matrix(G)
        K = np.empty((p, p), dtype=np.float64)
        self._use_current_stream()
        _check(self._lib.fa_gram(self._ctx, ptr, ldg, p, n, K.ctypes.data_as(ctypes.c_void_p)),
               "fa_gram")
        return K

    def fa_gram_begin(self, p: int, n: int) -> None:
        _check(self._lib.fa_gram_begin(self._ctx, int(p), int(n)), "fa_gram_begin")

    def fa_gram_update(self, G, i: int) -> None:
        """Gradient ``i`` (row i of the ``[p, n]`` buffer ``G``) has arrived."""
        ptr, ldg, p, n = self._matrix(G)
        self._use_current_stream()
        _check(self._lib.fa_gram_update(self._ctx, ptr, ldg, int(i)), "fa_gram_update")

    def fa_gram_update_rows(self, G, i: int, row0: int, nrows: int) -> None:
        """Elements ``[row0, row0 + nrows)`` of gradient ``i`` have arrived in ``G``."""
        ptr, ldg, p, n = self._matrix(G)
        self._use_current_stream()
        _check(self._lib.fa_gram_update_rows(self._ctx, ptr, ldg, int(i), int(row0), int(nrows)),
               "fa_gram_update_rows")

    def fa_aggregate_arrived(self, G, m: int, lam: float, iters: int, tol: float, out=None):
        ptr, ldg, p, n = self._matrix(G)
        torch = self._torch
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=G.device)
        if not out.is_cuda or out.dtype != torch.float32 or out.numel() != n or not out.is_contiguous():
            raise TypeError("out must be a contiguous float32 device tensor of n elements")
        self._use_current_stream()
        _check(self._lib.fa_aggregate_arrived(self._ctx, ptr, ldg, int(m), float(lam), int(iters),
                                              float(tol), ctypes.c_void_p(out.data_ptr())),
               "fa_aggregate_arrived")
        return out

    def fa_gram_async(self, G) -> None:
        ptr, ldg, p, n = self._matrix(G)
        self._use_current_stream()
        _check(self._lib.fa_gram_async(self._ctx, ptr, ldg, p, n), "fa_gram_async")

    def fa_irls(self, K: np.ndarray, m: int, lam: float, iters: int, tol: float) -> None:
        K = np.ascontiguousarray(K, dtype=np.float64)
        p = K.shape[0]
        if K.shape != (p, p):
            raise TypeError("K must be square")
        self._use_current_stream()
        _check(self._lib.fa_irls(self._ctx, K.ctypes.data_as(ctypes.c_void_p), p, int(m),
                                 float(lam), int(iters), float(tol)), "fa_irls")

    def fa_combine(self, G, c: np.ndarray, out=None):
        ptr, ldg, p, n = self._matrix(G)
        torch = self._torch
        c = np.ascontiguousarray(c, dtype=np.float64)
        if c.shape != (p,):
            raise TypeError("c must have p entries")
        if out is None:
            out = torch.empty(n, dtype=torch.float32, device=G.device)
        self._use_current_stream()
        _check(self._lib.fa_combine(self._ctx, ptr, ldg, p, n, c.ctypes.data_as(ctypes.c_void_p),
                                    ctypes.c_void_p(out.data_ptr())), "fa_combine")
        return out

    def fa_basis(self, G, m: int):
        """Y (as a ``[m, n]`` float32 tensor: row a is column a of Y) for the last solve, whose
        ``m`` this must be (the library refuses any other: FA_ERR_ARG)."""
        ptr, ldg, p, n = self._matrix(G)
        torch = self._torch
        ldy = (n + 3) // 4 * 4
        Y = torch.empty((m, ldy), dtype=torch.float32, device=G.device)
        self._use_current_stream()
        _check(self._lib.fa_basis(self._ctx, ptr, ldg, p, n, int(m),
                                  ctypes.c_void_p(Y.data_ptr()), ldy), "fa_basis")
        return Y[:, :n]

    def fa_check_basis(self, G, Y):
        """(Y^T Y, Y^T G) as float64 arrays of shapes (m, m) and (m, p), computed on the device
        in one pass; Y is an ``[m, n]`` float32 device tensor whose rows are the columns of the
        basis, as fa_basis returns it."""
        ptr, ldg, p, n = self._matrix(G)
        torch = self._torch
        if (not Y.is_cuda or Y.dim() != 2 or Y.dtype != torch.float32 or Y.shape[1] != n or
                Y.stride(1) != 1):
            raise TypeError("Y must be an [m, n] float32 device tensor with unit inner stride")
        m = int(Y.shape[0])
        ldy = int(Y.stride(0)) if m > 1 else n
        YtY = np.empty((m, m), dtype=np.float64)
        YtG = np.empty((m, p), dtype=np.float64)
        self._use_current_stream()
        _check(self._lib.fa_check_basis(self._ctx, ptr, ldg, p, n, ctypes.c_void_p(Y.data_ptr()),
                                        ldy, m, YtY.ctypes.data_as(ctypes.c_void_p),
                                        YtG.ctypes.data_as(ctypes.c_void_p)), "fa_check_basis")
        return YtY, YtG

    def fa_enqueue_kernel(self, which: int, G, m: int, lam: float, iters: int, tol: float,
                          out=None) -> None:
        ptr, ldg, p, n = self._matrix(G)
        self._use_current_stream()
        optr = ctypes.c_void_p(out.data_ptr()) if out is not None else None
        _check(self._lib.fa_enqueue_kernel(self._ctx, int(which), ptr, ldg, p, n, int(m),
                                           float(lam), int(iters), float(tol), optr),
               "fa_enqueue_kernel")

    def fa_set_profiling(self, enabled: bool) -> None:
        _check(self._lib.fa_set_profiling(self._ctx, 1 if enabled else 0), "fa_set_profiling")

    def fa_get_timings(self) -> np.ndarray:
        ms = (ctypes.c_float * 4)()
        _check(self._lib.fa_get_timings(self._ctx, ctypes.byref(ms)), "fa_get_timings")
        return np.array(list(ms), dtype=np.float64)
