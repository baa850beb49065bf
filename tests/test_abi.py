"""Host-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before touching a device.  No GPU needed."""
import ctypes
import os
import re

import pytest

from paper_2202_01085_amd import build, f3m

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(f3m.LIB_PATH):
        build.build_lib()
    return f3m.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "f3m.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(f3m_[a-z0-9_]+|direct_kmvm[a-z0-9_]*)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"f3m_plan", "f3m_plan_ex", "f3m_kmvm", "direct_kmvm", "direct_kmvm_rows_f64", "f3m_destroy",
            "f3m_last_error", "f3m_plan_info", "f3m_plan_get_perm", "f3m_plan_get_point_keys",
            "f3m_plan_get_boxes", "f3m_plan_get_list", "f3m_stage_times", "f3m_level_times", "f3m_plan_xy",
            "direct_kmvm_xy", "direct_kmvm_xy_rows_f64", "f3m_plan_source_info", "f3m_plan_get_source_perm",
            "f3m_plan_get_source_boxes", "f3m_cg_solve", "f3m_kmvm_multi", "f3m_trim_memory",
            "direct_kmvm_rows_f64_static"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_struct_sizes_match_the_header():
    assert ctypes.sizeof(f3m.Options) == 4 * 4 + 4 + 4 + 4 + 4
    assert ctypes.sizeof(f3m.Info) == 8 + 6 * 4 + 2 * 4 + 7 * 4 + 4 + 5 * 21 * 8 + 8 + 8 + 4 + 21 * 4 + 2 * 21 * 8
    assert ctypes.sizeof(f3m.Times) == 14 * 4
    assert ctypes.sizeof(f3m.SourceInfo) == 8 + 4 + 7 * 4 + 2 * 21 * 8


def test_argument_checks_need_no_device(lib):
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(4096)      # never dereferenced: every call below fails its checks first
    cases = [
        (fake, -1, 3, 1.0, 4, 2.0),   # n < 0
        (fake, 10, 0, 1.0, 4, 2.0),   # D out of range
        (fake, 10, 8, 1.0, 4, 2.0),
        (fake, 10, 3, 0.0, 4, 2.0),   # lengthscale
        (fake, 10, 3, float("inf"), 4, 2.0),
        (fake, 10, 3, 1.0, 1, 2.0),   # nodes
        (fake, 10, 3, 1.0, 4, 0.0),   # eta
        (None, 10, 3, 1.0, 4, 2.0),   # null X
    ]
    for X, n, D, g, p, eta in cases:
        assert lib.f3m_plan(X, n, D, g, p, eta, None, ctypes.byref(h)) == 1
        assert not h.value
        assert lib.f3m_last_error() != b""
    assert lib.f3m_plan(fake, 2 ** 31, 3, 1.0, 4, 2.0, None, ctypes.byref(h)) == 3
    assert lib.f3m_plan(fake, 10, 7, 1.0, 4, 2.0, None, ctypes.byref(h)) == 3      # 4^7 nodes
    assert lib.f3m_plan(fake, 10, 3, 1.0, 4, 2.0, None, None) == 1                 # null plan_out
    assert lib.f3m_kmvm(None, fake, fake, None) == 1
    assert lib.direct_kmvm(fake, 10, 3, 1.0, None, fake, None) == 1
    assert lib.direct_kmvm(fake, 10, 3, 1.0, fake, fake, None) == 1                # b aliases y
    assert lib.direct_kmvm(None, 0, 3, 1.0, None, None, None) == 0                 # empty problem
    # two point sets
    opt = None
    assert lib.f3m_plan_xy(fake, 10, None, 5, 3, 1.0, 4, 2.0, opt, None, ctypes.byref(h)) == 1   # null Y
    assert lib.f3m_plan_xy(fake, 10, fake, -1, 3, 1.0, 4, 2.0, opt, None, ctypes.byref(h)) == 1  # ny < 0
    assert lib.f3m_plan_xy(fake, 10, fake, 2 ** 31, 3, 1.0, 4, 2.0, opt, None, ctypes.byref(h)) == 3
    assert lib.f3m_plan_xy(None, 10, fake, 5, 3, 1.0, 4, 2.0, opt, None, ctypes.byref(h)) == 1   # null X
    assert not h.value
    assert lib.direct_kmvm_xy(fake, 10, None, 5, 3, 1.0, fake, fake, None) == 1                  # null Y
    assert lib.direct_kmvm_xy(fake, 10, fake, 5, 3, 1.0, fake, fake, None) == 1                  # b aliases y
    assert lib.direct_kmvm_xy(None, 0, fake, 5, 3, 1.0, fake, None, None) == 0                   # no targets
    assert lib.direct_kmvm_xy_rows_f64(fake, 10, fake, 5, 3, 1.0, fake, None, 4, fake, None) == 1  # null rows
    # the entry point that allocates nothing refuses what its static scratch cannot hold, before any device call
    assert lib.direct_kmvm_rows_f64_static(fake, 10, 3, 1.0, fake, fake, 16385, fake, None) == 3
    assert b"16384" in lib.f3m_last_error()
    assert lib.direct_kmvm_rows_f64_static(fake, 10, 3, 1.0, fake, None, 4, fake, None) == 1     # null rows
    assert lib.direct_kmvm_rows_f64_static(fake, 10, 3, 1.0, fake, fake, 0, fake, None) == 0     # no rows
    assert lib.f3m_kmvm_multi(None, fake, 10, fake, 10, 2, None) == 1                            # null plan
    it = ctypes.c_int(-1)
    assert lib.f3m_cg_solve(None, 1.0, fake, fake, 10, 1e-6, ctypes.byref(it), None, None) == 1   # null plan
    assert it.value == 0
    lib.f3m_destroy(None)                                                           # allowed
