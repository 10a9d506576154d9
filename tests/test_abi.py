"""The C-ABI library builds, loads without a GPU, and exports what include/fa.h declares."""
import ctypes
import os
import re
import subprocess

import pytest

import paper_2302_05865_amd as fa
from paper_2302_05865_amd import _ctypes_defs as defs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fa.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(fa_[a-z_]+)\s*\(", text)
    return sorted(set(names))


def test_library_is_built_and_loads():
    assert os.path.exists(fa.library_path()), "run python -m paper_2302_05865_amd.build"
    lib = fa.load_library()
    assert b"gfx950" in lib.fa_version()


def test_every_declared_symbol_is_exported_and_bound():
    lib = fa.load_library()
    declared = _declared_functions()
    assert len(declared) >= 12
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in fa.h but not exported"
    assert sorted(fa.EXPORTED_SYMBOLS) == declared


def test_status_strings():
    lib = fa.load_library()
    seen = {lib.fa_status_string(k) for k in range(7)}
    assert len(seen) == 7 and all(s for s in seen)


def test_struct_layouts_match_the_header(tmp_path):
    src = tmp_path / "layout.c"
    src.write_text(r'''
#include <stdio.h>
#include <stddef.h>
#include "fa.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %d %d\n", sizeof(fa_config),
         sizeof(fa_info),
         offsetof(fa_info, objective), offsetof(fa_info, s), offsetof(fa_info, c),
         offsetof(fa_info, A), offsetof(fa_info, K), offsetof(fa_config, clamp_delta),
         offsetof(fa_config, exponent_a), offsetof(fa_config, layout),
         offsetof(fa_config, solver), offsetof(fa_config, wide_spin_budget),
         offsetof(fa_config, gram), FA_P_MAX, FA_ITERS_MAX);
  return 0;
}''')
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    vals = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    I, C = defs.FaInfo, defs.FaConfig
    assert vals == [ctypes.sizeof(C), ctypes.sizeof(I), I.objective.offset, I.s.offset,
                    I.c.offset, I.A.offset, I.K.offset, C.clamp_delta.offset,
                    C.exponent_a.offset, C.layout.offset, C.solver.offset,
                    C.wide_spin_budget.offset, C.gram.offset, defs.FA_P_MAX, defs.FA_ITERS_MAX]


def test_default_config_needs_no_gpu():
    lib = fa.load_library()
    cfg = defs.FaConfig()
    lib.fa_default_config(ctypes.byref(cfg))
    assert cfg.p_max == 64 and cfg.dtype == defs.FA_F32
    assert cfg.clamp_delta == 1e-6 and cfg.rank_tol == 1e-12 and cfg.pair_tol == 1e-12
    assert cfg.exponent_a == 2.0 and cfg.layout == defs.FA_WORKER_MAJOR
    assert cfg.solver == defs.FA_SOLVER_AUTO and cfg.wide_spin_budget == 1 << 22
    assert cfg.gram == defs.FA_GRAM_AUTO


def test_argument_errors_are_synchronous_without_a_context():
    """NULL context / NULL pointers are rejected before any HIP call."""
    lib = fa.load_library()
    assert lib.fa_aggregate(None, None, 0, 1, 1, 1, 0.0, 1, 0.0, None) == defs.FA_ERR_ARG
    assert lib.fa_get_info(None, None) == defs.FA_ERR_ARG
    assert lib.fa_gram(None, None, 0, 1, 1, None) == defs.FA_ERR_ARG
    assert lib.fa_set_profiling(None, 1) == defs.FA_ERR_ARG
    ctx = ctypes.c_void_p()
    bad = defs.FaConfig()
    lib.fa_default_config(ctypes.byref(bad))      # n_max = 0 is invalid
    assert lib.fa_create(ctypes.byref(bad), ctypes.byref(ctx)) == defs.FA_ERR_ARG
    bad.n_max = 10
    bad.p_max = 65
    assert lib.fa_create(ctypes.byref(bad), ctypes.byref(ctx)) == defs.FA_ERR_ARG
    bad.p_max = 8
    bad.exponent_a = 0.5          # the terms must stay concave: a >= 1
    assert lib.fa_create(ctypes.byref(bad), ctypes.byref(ctx)) == defs.FA_ERR_ARG
    bad.exponent_a = 2.0
    bad.solver = 3                # no such solver
    assert lib.fa_create(ctypes.byref(bad), ctypes.byref(ctx)) == defs.FA_ERR_ARG
    bad.solver = defs.FA_SOLVER_AUTO
    bad.wide_spin_budget = -1
    assert lib.fa_create(ctypes.byref(bad), ctypes.byref(ctx)) == defs.FA_ERR_ARG
    bad.wide_spin_budget = 0
    bad.gram = 3                  # no such accumulation mode
    assert lib.fa_create(ctypes.byref(bad), ctypes.byref(ctx)) == defs.FA_ERR_ARG
    assert lib.fa_basis(None, None, 0, 1, 1, 1, None, 0) == defs.FA_ERR_ARG
    # the entry point without a context: its size limit and its argument checks come before
    # any HIP call
    assert lib.fa_aggregate_static(None, 0, 65, 1, 0, 1, 0.0, 1, 0.0, None, None) == \
        defs.FA_ERR_TOO_LARGE
    assert lib.fa_aggregate_static(None, 0, 4, 1, 0, 1, 0.0, 1, 0.0, None, None) == defs.FA_ERR_ARG
    assert lib.fa_aggregate_static(None, 0, 4, 1, 7, 1, 0.0, 1, 0.0, None, None) == defs.FA_ERR_ARG
    lib.fa_destroy(None)
