"""CPU-only checks of the C ABI: the built library loads, exports every function the header
declares, and rejects bad arguments without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fvdb_hotpath.h")
LIB = os.path.join(ROOT, "paper_2407_01781_amd", "libfvdb_hotpath.so")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fx_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2407_01781_amd import build
        build.build()
    return C.CDLL(LIB)


def test_header_declares_the_three_calls_of_the_path():
    names = _declared_functions()
    for n in ("fx_build_index_grid", "fx_build_kernel_map", "fx_sparse_conv_fwd"):
        assert n in names


def test_every_declared_symbol_is_exported(lib):
    for n in _declared_functions():
        assert hasattr(lib, n), n


def test_bad_arguments_are_rejected_on_the_host(lib):
    lib.fx_last_error.restype = C.c_char_p
    h = C.c_void_p()
    assert lib.fx_build_index_grid(None, C.c_int64(-1), None, 0, None, C.byref(h)) == -1
    assert b"fx_build_index_grid" in lib.fx_last_error()
    assert lib.fx_build_index_grid(None, C.c_int64(0), None, 0, None, None) == -1
    jo = (C.c_int64 * 4)(0, 5, 3, 8)        # overlapping ranges
    dummy = C.c_void_p(256)
    assert lib.fx_build_index_grid(dummy, C.c_int64(8), jo, 2, None, C.byref(h)) == -1
    jo = (C.c_int64 * 2)(0, 9)              # beyond n_rows
    assert lib.fx_build_index_grid(dummy, C.c_int64(8), jo, 1, None, C.byref(h)) == -1
    assert lib.fx_grid_info(None, None, None, None, None) == -1
    assert lib.fx_build_kernel_map(None, 3, 1, None, None, None) == -1
    assert lib.fx_sparse_conv_fwd(None, None, 0, None, 4, 4, None, 0, None) == -1
    assert lib.fx_kmap_info(None, None, None, None, None) == -1
    # backward pass, transposed convolution, pooling, upsampling, subdivision: null handles / pointers
    assert lib.fx_sparse_conv_bwd_data(None, None, 0, None, 4, 4, None, 0, None) == -1
    assert lib.fx_sparse_conv_bwd_weight(None, None, None, 0, 4, 4, None, 0, None) == -1
    assert lib.fx_sparse_conv_transpose_fwd(None, None, 0, None, 4, 4, None, 0, None) == -1
    assert lib.fx_pool2(None, 0, None, 0, 4, None, None) == -1
    assert lib.fx_upsample2(None, None, 0, 4, None, None) == -1
    assert lib.fx_pool2_bwd(None, 0, None, None, 0, 4, None, None) == -1
    assert lib.fx_upsample2_bwd(None, None, 0, 4, None, None) == -1
    assert lib.fx_grid_subdivide2(None, None, None) == -1
    assert b"fx_grid_subdivide2" in lib.fx_last_error()
    assert lib.fx_sparse_conv_leaf_fwd(None, None, 0, None, 8, 16, None, 0, None) == -1
    assert b"fx_sparse_conv_leaf_fwd" in lib.fx_last_error()
    assert lib.fx_sparse_conv_leaf_bwd_data(None, None, 0, None, 16, 8, None, 0, None) == -1
    assert b"fx_sparse_conv_leaf_bwd_data" in lib.fx_last_error()
    assert lib.fx_sparse_conv_leaf_bwd_weight(None, None, None, 0, 8, 16, None, 0, None) == -1
    assert b"fx_sparse_conv_leaf_bwd_weight" in lib.fx_last_error()
    assert lib.fx_grid_pad(None, 1, None, None) == -1
    assert b"fx_grid_pad" in lib.fx_last_error()
    assert lib.fx_build_kernel_map_onto(None, None, 3, None, None) == -1
    assert b"fx_build_kernel_map_onto" in lib.fx_last_error()
    # grid from points: null origin / voxel size, non-positive or non-finite voxel size
    f3 = C.c_float * 3
    assert lib.fx_build_index_grid_from_points(None, C.c_int64(0), None, 0, None, None, None, C.byref(h)) == -1
    assert lib.fx_build_index_grid_from_points(None, C.c_int64(0), None, 0, f3(0, 0, 0), f3(1, 0, 1), None,
                                               C.byref(h)) == -1
    assert lib.fx_build_index_grid_from_points(None, C.c_int64(0), None, 0, f3(0, 0, 0), f3(1, float("inf"), 1), None,
                                               C.byref(h)) == -1
    assert b"voxel sizes" in lib.fx_last_error()


def test_leaf_record_is_96_bytes_with_an_80_byte_payload():
    from paper_2407_01781_amd.binding import LEAF_DTYPE
    assert LEAF_DTYPE.itemsize == 96 and LEAF_DTYPE.fields["origin"][1] == 80


def test_options_and_allocator_hook_on_the_host(lib):
    lib.fx_last_error.restype = C.c_char_p
    v = C.c_int32(7)
    assert lib.fx_get_option(b"leaf_dispatch", C.byref(v)) == 0 and v.value == -1          # automatic by default
    assert lib.fx_set_option(b"leaf_dispatch", 0) == 0
    assert lib.fx_get_option(b"leaf_dispatch", C.byref(v)) == 0 and v.value == 0
    assert lib.fx_set_option(b"leaf_dispatch", -1) == 0
    assert lib.fx_set_option(b"no_such_switch", 1) == -1 and b"no_such_switch" in lib.fx_last_error()
    assert lib.fx_set_option(b"cache_mb", -2) == -1 and lib.fx_set_option(None, 1) == -1
    assert lib.fx_get_option(b"cache_mb", None) == -1
    cb = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p)(lambda n, s, c: None)
    assert lib.fx_set_allocator(C.cast(cb, C.c_void_p), None, None) == -1             # both functions or neither
    assert lib.fx_set_allocator(None, None, None) == 0
