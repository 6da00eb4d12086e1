"""mqg_gather_features_static, the gather for callers that cannot allocate, through the C ABI.

Its rows and stats must equal those of mqg_gather_features byte for byte (and the oracle's),
on calls in a row that share the library's fixed device array: the second call is smaller than
the first, so whatever the first left in the lists and counters must not leak into it.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2601_04707_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mqg():
    from paper_2601_04707_amd import mqg as m
    assert torch.cuda.is_available()
    return m


def gather_both(mqg, ctx, cache, ids_np, idx_dtype, cap, dim, dtype, stride):
    """(rows, stats) of the context gather and of the static gather for the same ids."""
    count = len(ids_np)
    ids = torch.zeros(cap, dtype=idx_dtype, device="cuda")
    ids[:count] = torch.from_numpy(ids_np).to(idx_dtype).cuda()
    num = torch.tensor([count], dtype=torch.int64, device="cuda")
    res = []
    for static in (False, True):
        buf = torch.full((cap, stride), 7.0, dtype=dtype, device="cuda")
        stats = torch.full((2,), -1, dtype=torch.int64, device="cuda")
        if static:
            mqg.mqg_gather_features_static(cache, ids, num, buf[:, :dim], stats)
        else:
            mqg.mqg_gather_features(ctx, cache, ids, num, buf[:, :dim], stats)
        torch.cuda.synchronize()
        assert torch.all(buf[count:] == 7.0)                       # rows past the count stay untouched
        res.append((buf[:count, :dim].contiguous().cpu().numpy(), stats.tolist()))
    return res


@pytest.mark.parametrize("dim,dtype,idx_dtype", [(602, torch.float32, torch.int64), (100, torch.float32, torch.int32),
                                                 (128, torch.float16, torch.int64)])
def test_static_gather_equals_context_gather_on_calls_in_a_row(mqg, dim, dtype, idx_dtype):
    n = 30_000
    rp, ci = synth.chung_lu_graph(n, 500_000, max_degree=2500, seed=5)
    g = mqg.Graph(rp.cuda(), ci.cuda())
    feats = synth.node_features(n, dim, dtype=dtype, seed=7).pin_memory()
    elt = feats.element_size()
    stride = (dim * elt + 63) // 64 * 64 // elt
    ctx = mqg.Context(g, 1024, [25])
    cache = mqg.Cache(g, feats, n * 3 // 10, cache_stride=stride)
    mqg.mqg_build_cache(ctx, g, cache)
    want = oracle.build_cache(rp.numpy(), n * 3 // 10, feats.numpy())
    rng = np.random.default_rng(11)
    # a large call, a smaller one, an empty one, a large one again: each must be right on its own
    for count in (21_000, 1_300, 0, 17_777):
        ids_np = rng.permutation(n)[:count].astype(np.int64)
        (rows_ctx, stats_ctx), (rows_st, stats_st) = gather_both(mqg, ctx, cache, ids_np, idx_dtype, count + 3, dim, dtype,
                                                                 stride)
        ref, h, m = oracle.gather(ids_np, feats.numpy(), want)
        assert rows_st.tobytes() == rows_ctx.tobytes(), count
        assert rows_st.tobytes() == ref.tobytes(), count
        assert stats_st == stats_ctx == [h, m], count


def test_static_gather_without_a_cache_and_its_limit(mqg):
    n, dim = 5_000, 64
    rp, ci = synth.chung_lu_graph(n, 60_000, max_degree=500, seed=2)
    g = mqg.Graph(rp.cuda(), ci.cuda())
    feats = synth.node_features(n, dim, seed=3).cuda()
    ids_np = np.random.default_rng(0).permutation(n)[:3_000].astype(np.int64)
    ids = torch.from_numpy(ids_np).cuda()
    num = torch.tensor([3_000], dtype=torch.int64, device="cuda")
    out = torch.zeros((3_000, dim), dtype=torch.float32, device="cuda")
    stats = torch.zeros(2, dtype=torch.int64, device="cuda")
    mqg.mqg_gather_features_static(mqg.Cache(g, feats, None), ids, num, out, stats)     # no cache: rows straight from feats
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), feats.cpu().numpy()[ids_np])
    assert stats.tolist() == [0, 3_000]
    # with a cache, more ids than the fixed array holds are refused before anything is enqueued
    ctx = mqg.Context(g, 16, [2])
    cache = mqg.Cache(g, feats, n // 2)
    mqg.mqg_build_cache(ctx, g, cache)
    too_many = mqg.MQG_GATHER_STATIC_MAX_IDS + 1
    rc = mqg.lib.mqg_gather_features_static(ctypes.byref(cache.c), mqg.MQG_I64, ids.data_ptr(), num.data_ptr(), too_many,
                                            out.data_ptr(), dim, None, None)
    assert rc == mqg.MQG_ERR_CAPACITY
    assert b"MQG_GATHER_STATIC_MAX_IDS" in mqg.lib.mqg_last_error(None)
    assert mqg.lib.mqg_gather_features_static(None, mqg.MQG_I64, None, None, 0, None, 0, None, None) == mqg.MQG_ERR_INVALID_ARG
