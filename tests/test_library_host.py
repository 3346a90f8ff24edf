"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, sizes workspaces sanely and rejects bad
arguments with codes before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2211_13878_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2211_13878_amd.build import build_library
        build_library()
    return binding.load_library()


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "galv_dp.h")).read()
    declared = set(re.findall(r"\b(galv_(?:dp|alg1)_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_workspace_bytes_covers_tables(lib):
    for (B, L, S, E) in [(1, 4, 6, 256), (8, 32, 22, 16384), (64, 96, 44, 32768),
                         (16, 128, 128, 65536), (1, 1, 1, 0)]:
        n = binding.galv_dp_workspace_bytes(binding.make_desc(B, L, S, E))
        need = B * S * (E + 1) * (4 * (L - 1) + 16)          # back-pointers + two cost rows
        assert need <= n <= 1.6 * need + (1 << 22)


@pytest.mark.parametrize("args", [(0, 4, 6, 256, 1), (1, 0, 6, 256, 1), (1, 4, 0, 256, 1),
                                  (1, 4, 6, -1, 1), (1, 4, 6, 256, 0), (1, 4, 2000, 256, 1)])
def test_bad_desc_is_invalid_arg(lib, args):
    with pytest.raises(binding.GalvError) as ei:
        binding.galv_dp_workspace_bytes(binding.make_desc(*args))
    assert ei.value.code == binding.GALV_ERR_INVALID_ARG
    assert binding.galv_dp_last_error() != ""


def test_unknown_flag_and_range(lib):
    with pytest.raises(binding.GalvError) as ei:
        binding.galv_dp_workspace_bytes(binding.make_desc(1, 4, 6, 256, 1, flags=0x4000))
    assert ei.value.code == binding.GALV_ERR_INVALID_ARG
    with pytest.raises(binding.GalvError) as ei:
        binding.galv_dp_workspace_bytes(binding.make_desc(1, 4, 6, (1 << 30) + 1, 1))
    assert ei.value.code == binding.GALV_ERR_RANGE


def test_create_rejects_null_small_and_misaligned_workspace(lib):
    desc = binding.make_desc(1, 4, 6, 256)
    h = ctypes.c_void_p(None)
    rc = lib.galv_dp_create(ctypes.byref(desc), None, 1 << 30, ctypes.byref(h))
    assert rc == binding.GALV_ERR_WORKSPACE and not h.value
    rc = lib.galv_dp_create(ctypes.byref(desc), ctypes.c_void_p(4096), 16, ctypes.byref(h))
    assert rc == binding.GALV_ERR_WORKSPACE and "smaller" in binding.galv_dp_last_error()
    rc = lib.galv_dp_create(ctypes.byref(desc), ctypes.c_void_p(4097), 1 << 30, ctypes.byref(h))
    assert rc == binding.GALV_ERR_WORKSPACE
    rc = lib.galv_dp_create(ctypes.byref(desc), ctypes.c_void_p(4096), 1 << 30, None)
    assert rc == binding.GALV_ERR_INVALID_ARG


def test_null_handle_calls(lib):
    assert lib.galv_dp_solve_batched(*([None] * 9)) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_dp_backtrack(None, None, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_dp_export_tables(None, 0, None, None, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_dp_get_status(None, None, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_dp_best_per_budget(None, None, None, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_dp_backtrack_queries(None, 1, None, None, None, None, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_dp_destroy(None) == binding.GALV_OK


def test_alg1_reduce_rejects_bad_host_arguments(lib):
    deg = (ctypes.c_int32 * 2)(1, 2)
    one = ctypes.c_void_p(256)          # never dereferenced: every call below fails before a launch
    assert lib.galv_alg1_reduce(0, 2, deg, one, one, 0, 1, one, one, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_alg1_reduce(1, 0, deg, one, one, 0, 1, one, one, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_alg1_reduce(1, 17, deg, one, one, 0, 1, one, one, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_alg1_reduce(1, 2, None, one, one, 0, 1, one, one, None) == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_alg1_reduce(1, 2, deg, None, one, 0, 1, one, one, None) == binding.GALV_ERR_INVALID_ARG
    bad = (ctypes.c_int32 * 2)(1, 0)
    assert lib.galv_alg1_reduce(1, 2, bad, one, one, 0, 1, one, one, None) == binding.GALV_ERR_INVALID_ARG
    assert "pp_degree" in binding.galv_dp_last_error()


def test_one_byte_back_pointers_need_few_strategies(lib):
    n = ctypes.c_size_t(0)
    ok = binding.make_desc(1, 4, 255, 256, flags=binding.GALV_DP_BP_U8)
    assert lib.galv_dp_workspace_bytes(ctypes.byref(ok), ctypes.byref(n)) == binding.GALV_OK
    bad = binding.make_desc(1, 4, 256, 256, flags=binding.GALV_DP_BP_U8)
    assert lib.galv_dp_workspace_bytes(ctypes.byref(bad), ctypes.byref(n)) == binding.GALV_ERR_INVALID_ARG
    assert "255" in binding.galv_dp_last_error()
    unknown = binding.make_desc(1, 4, 6, 256, flags=0x4000)
    assert lib.galv_dp_workspace_bytes(ctypes.byref(unknown), ctypes.byref(n)) == binding.GALV_ERR_INVALID_ARG
