"""CPU-only checks of the boundary: the library builds, loads and exports every symbol that
include/tv.h declares; argument errors come back as negative codes without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2209_12708_amd", "lib", "libtv.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    src = open(os.path.join(ROOT, "include", "tv.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tv_[a-z_0-9]+)\s*\(", src)))


def test_header_declares_the_expected_calls():
    names = declared_functions()
    for must in ("tv_model_create", "tv_model_destroy", "tv_workspace_query", "tv_verify", "tv_certify",
                 "tv_last_error", "tv_version"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"libtv.so lacks {name}"


def test_binding_lists_the_same_symbols():
    from paper_2209_12708_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()


def test_argument_errors_without_gpu(lib):
    lib.tv_last_error.restype = ctypes.c_char_p
    lib.tv_version.restype = ctypes.c_char_p
    assert b"gfx950" in lib.tv_version()
    assert lib.tv_model_create(None, None, None) == -1
    assert b"null" in lib.tv_last_error()
    assert lib.tv_workspace_query(None, 1, 8, 1, None, None) == -1
    assert lib.tv_verify(*([None] * 17)) == -1
    assert lib.tv_op_concretize(None, None, 1, 1, 4, 1, 4, 1, 2, None, None, None, None) == -1
    one = ctypes.c_void_p(16)   # non-null dummy: shape checks come before any launch
    assert lib.tv_op_concretize(one, one, 1, 1, 4, 1, 6, 1, 2, one, one, one, None) == -2     # n % 4 != 0
    assert lib.tv_op_concretize(one, one, 1, 1, 4, 1, 8, 1, 7, one, one, one, None) == -3     # bad norm
    assert lib.tv_verify_padded(*([None] * 18)) == -1 and lib.tv_certify_padded(*([None] * 18)) == -1
    # tile search entry points: the candidate table and the built-in rule are host logic
    lib.tv_affine_tile_default.argtypes = [ctypes.c_longlong, ctypes.c_int, ctypes.c_int]
    n_tiles = lib.tv_affine_tile_count()
    assert n_tiles >= 4
    for M, N, K in ((2080, 64, 64), (2080, 192, 64), (132096, 128, 256), (1050624, 768, 256)):
        assert 0 <= lib.tv_affine_tile_default(M, N, K) < n_tiles
    assert lib.tv_affine_tile_default(0, 8, 8) == -2
    assert lib.tv_op_affine_split_tile(one, 1, 1, 4, 1, 8, 8, one, None, one, n_tiles, None) == -6
    assert lib.tv_op_affine_split_tile(one, 1, 1, 4, 1, 6, 8, one, None, one, 0, None) == -2      # K % 8 != 0
