"""The C-ABI library loads without a GPU and exports every function include/mqg.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mqg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mqg_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_operations():
    names = declared_functions()
    for must in ("mqg_build_cache", "mqg_sample_blocks", "mqg_gather_features", "mqg_sage_mean_aggregate",
                 "mqg_ctx_create", "mqg_ctx_destroy", "mqg_last_error"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2601_04707_amd import mqg
    for name in declared_functions():
        assert hasattr(mqg.lib, name), name
    assert sorted(mqg.EXPORTS) == declared_functions()
    assert mqg.lib.mqg_version() >= 100


def test_struct_layouts_match_the_header():
    from paper_2601_04707_amd import mqg
    assert ctypes.sizeof(mqg.CGraph) == 8 + 8 + 4 + 4 + 8 + 8
    assert ctypes.sizeof(mqg.CCache) == 8 + 8 + 4 + 4 + 8 * 6
    assert ctypes.sizeof(mqg.CBlock) == 8 * 7
    assert mqg.CCache.feats.offset == 24 and mqg.CCache.cached_ids.offset == 64


def test_null_arguments_are_refused_without_touching_a_gpu():
    from paper_2601_04707_amd import mqg
    assert mqg.lib.mqg_ctx_create(None, None, 1, None, 1) == mqg.MQG_ERR_INVALID_ARG
    h = ctypes.c_void_p()
    assert mqg.lib.mqg_ctx_create(ctypes.byref(h), None, 1, None, 1) == mqg.MQG_ERR_INVALID_ARG
    assert b"NULL" in mqg.lib.mqg_last_error(None)
    assert mqg.lib.mqg_ctx_destroy(None) == mqg.MQG_OK
    assert mqg.lib.mqg_sample_blocks(None, None, None, 0, None, 0, 0, None, None) == mqg.MQG_ERR_INVALID_ARG
    assert mqg.lib.mqg_gather_features(None, None, 0, None, None, 0, None, 0, None, None) == mqg.MQG_ERR_INVALID_ARG
    assert mqg.lib.mqg_sage_mean_aggregate(None, None, None, 0, None, 0, 1, 0, None) == mqg.MQG_ERR_INVALID_ARG
    assert mqg.lib.mqg_build_cache(None, None, None, None) == mqg.MQG_ERR_INVALID_ARG


def test_block_bounds_follow_the_documented_formula():
    from paper_2601_04707_amd import mqg
    b = mqg.block_bounds(10_000, 256, [10, 5])
    assert b[1] == (256, 256 + 1280, 1280)
    assert b[0] == (1536, 10_000, 15_360)
    b = mqg.block_bounds(2_449_029, 1024, [15, 10, 5])
    assert b[2] == (1024, 6144, 5120) and b[1] == (6144, 67_584, 61_440) and b[0] == (67_584, 1_081_344, 1_013_760)
