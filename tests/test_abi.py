"""CPU-side checks of the boundary: the in-tree library loads and exports every symbol the header declares,
and the Python binding names the same entry points.  No compute calls (no GPU here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sp_conv.h")
LIB = os.path.join(ROOT, "paper_2012_13846_amd", "libsp_conv.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sp_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_north_star_entry_points():
    names = declared_functions()
    for must in ("sp_coords_build", "sp_kmap_build", "sp_conv_fwd", "sp_conv_bwd_data", "sp_conv_bwd_weight",
                 "sp_kmap_transpose"):
        assert must in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} is not built: run python -m paper_2012_13846_amd.build")
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in sp_conv.h but not exported"
    lib.sp_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.sp_version()


def test_binding_has_the_same_names():
    from paper_2012_13846_amd import binding
    for name in ("sp_coords_build", "sp_kmap_build", "sp_kmap_transpose", "sp_conv_fwd", "sp_conv_bwd_data",
                 "sp_conv_bwd_weight", "sp_pool_trim", "sp_pool_bytes", "sp_version"):
        assert callable(getattr(binding, name))


def test_host_side_argument_checks_need_no_gpu():
    lib = ctypes.CDLL(LIB)
    lib.sp_last_error.restype = ctypes.c_char_p
    out = ctypes.c_void_p()
    # negative size, NULL out pointer, bad stride: rejected before any device call
    assert lib.sp_coords_build(None, ctypes.c_int64(-1), 1, None, ctypes.byref(out)) == -1
    assert lib.sp_coords_build(None, ctypes.c_int64(0), 1, None, None) == -1
    assert lib.sp_coords_build(None, ctypes.c_int64(0), 0, None, ctypes.byref(out)) == -1
    assert lib.sp_coords_build(None, ctypes.c_int64(5), 1, None, ctypes.byref(out)) == -1
    assert b"NULL" in lib.sp_last_error()
    assert lib.sp_kmap_build(None, 3, 1, 1, None, ctypes.byref(out), None) == -1
    assert lib.sp_conv_fwd(None, None, None, None, 16, 16, 0, None) == -1
    assert lib.sp_conv_bwd_data(None, None, None, None, 16, 16, 0, None) == -1
    assert lib.sp_conv_bwd_weight(None, None, None, None, 16, 16, 0, None) == -1
    assert lib.sp_kmap_destroy(None) == 0 and lib.sp_coords_destroy(None) == 0
