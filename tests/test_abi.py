"""CPU-side checks of the boundary: the library builds for gfx950, loads, and exports exactly
what include/gpws.h declares.  No kernel is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2405_18328_amd", "libgpws.so")
HEADER = os.path.join(ROOT, "include", "gpws.h")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(gp_[a-z_0-9]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import sys
        sys.path.insert(0, ROOT)
        from paper_2405_18328_amd.build import build_library
        build_library(verbose=False)
    return ctypes.CDLL(LIB)


def test_header_declares_the_named_entry_points():
    names = _declared()
    for must in ("gp_kmv", "gp_cg_solve", "gp_mll_grad", "gp_create", "gp_destroy", "gp_set_theta"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in _declared():
        assert hasattr(lib, name), f"{name} declared in gpws.h but not exported"


def test_binding_mirrors_the_header(lib):
    from paper_2405_18328_amd import binding
    assert sorted(binding.EXPORTS) == _declared()
    for name in _declared():
        assert callable(getattr(binding, name))
    src = open(HEADER).read()
    for const in ("GP_MAX_D", "GP_MAX_T"):
        assert int(re.search(rf"#define {const} (\d+)", src).group(1)) == getattr(binding, const)


def test_null_context_calls_fail_cleanly_without_a_gpu(lib):
    lib.gp_last_error.restype = ctypes.c_char_p
    assert lib.gp_destroy(None) == 0
    assert lib.gp_set_theta(None, None, ctypes.c_double(1.0), ctypes.c_double(1.0)) == -1
    assert lib.gp_kmv(None, None, ctypes.c_int64(1), 1, None, ctypes.c_int64(1), 0) == -1
    lib.gp_workspace_bytes.restype = ctypes.c_size_t
    assert lib.gp_workspace_bytes(None, 4) == 0
    assert lib.gp_last_error(None) == b"NULL context"
    out = ctypes.c_void_p()
    # argument errors are reported before any HIP call
    assert lib.gp_create(ctypes.byref(out), 7, ctypes.c_int64(10), 2, ctypes.c_void_p(16), None) == -1
    assert lib.gp_create(ctypes.byref(out), 0, ctypes.c_int64(0), 2, ctypes.c_void_p(16), None) == -1
    assert lib.gp_create(ctypes.byref(out), 0, ctypes.c_int64(10), 127, ctypes.c_void_p(16), None) == -1
    assert lib.gp_create(ctypes.byref(out), 0, ctypes.c_int64(10), 2, None, None) == -1
