"""HIP path versus CPU oracle, through the C ABI, on the same seeded inputs.

Bit-exact: sampled blocks (sizes, src_ids, indptr, indices), cache tables, gathered rows.
Aggregation: |gpu - oracle| <= tol * max(|oracle|, mean|x|), tol = 1e-5 (fp32), 2e-3 (fp16).
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from paper_2601_04707_amd import synth
from gpu_util import agg_tolerance_ok, assert_blocks_equal, hip_sample, to_dev

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float16: 2e-3}


@pytest.fixture(scope="module")
def mqg():
    from paper_2601_04707_amd import mqg as m
    assert torch.cuda.is_available()
    return m


def hub_graph(n=20000, edges=400_000, max_degree=3000, seed=1, ptr=torch.int64, idx=torch.int64):
    rp, ci = synth.chung_lu_graph(n, edges, max_degree=max_degree, seed=seed, ptr_dtype=ptr, idx_dtype=idx)
    return rp, ci


def run_aggregate_chain(mqg, ctx, blocks, x0_dev, want_blocks, feats_np_rows, dtype):
    """Per layer: GPU aggregate fed with the oracle's input of that layer, compared to the oracle."""
    L = len(want_blocks)
    h_ref = feats_np_rows
    for l in range(L):
        ref = oracle.mean_aggregate(want_blocks[l].indptr, want_blocks[l].indices, h_ref)
        x_dev = to_dev(torch.from_numpy(h_ref)) if l > 0 else x0_dev
        out = torch.empty((blocks.bounds[l][0], h_ref.shape[1]), dtype=x_dev.dtype, device="cuda")
        mqg.mqg_sage_mean_aggregate(ctx, blocks, l, x_dev, out)
        torch.cuda.synchronize()
        got = out[:want_blocks[l].num_dst].cpu().numpy()
        ok, worst = agg_tolerance_ok(got, ref, float(np.abs(h_ref.astype(np.float64)).mean()), TOL[dtype])
        assert ok, f"layer {l}: worst error/bound {worst}"
        h_ref = ref
    return h_ref


# ------------------------------------------------------------------------- config 1, whole path

def test_tiny_config_all_batches(mqg):
    w = synth.WORKLOADS["tiny"]
    rp, ci = synth.build_graph(w, seed=0)
    assert rp.dtype == torch.int32 and ci.dtype == torch.int32
    feats = synth.node_features(w.num_nodes, w.dim, dtype=w.feat_dtype, seed=1)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    ctx = mqg.Context(g, w.batch, w.fanouts)
    blocks = mqg.Blocks(g, w.batch, w.fanouts)
    cache = mqg.Cache(g, to_dev(feats), None)                     # all features in HBM, no cache
    feats_np = feats.numpy()
    rp_np, ci_np = rp.numpy(), ci.numpy()
    total_edges = 0
    for b, seeds in enumerate(synth.seed_batches(w.num_nodes, w.batch, 16, seed=2)):
        rng_seed = 1000 + b
        got = hip_sample(mqg, ctx, g, blocks, seeds, w.fanouts, rng_seed)
        want = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), w.fanouts, rng_seed)
        assert_blocks_equal(got, want)
        total_edges += sum(x.nnz for x in want)
        cap = blocks.bounds[0][1]
        x0 = torch.zeros((cap, w.dim), dtype=w.feat_dtype, device="cuda")
        stats = torch.zeros(2, dtype=torch.int64, device="cuda")
        mqg.mqg_gather_features(ctx, cache, blocks.src_ids[0], blocks.sizes[0, 1:2], x0, stats)
        torch.cuda.synchronize()
        ref_rows, _, _ = oracle.gather(want[0].src_ids, feats_np, None)
        ns = want[0].num_src
        assert x0[:ns].cpu().numpy().tobytes() == ref_rows.tobytes()
        assert torch.all(x0[ns:] == 0)                            # nothing written past num_src
        assert stats.tolist() == [0, ns]
        run_aggregate_chain(mqg, ctx, blocks, x0, want, ref_rows, np.float32)
    assert total_edges > 16 * 256 * 5


# ------------------------------------------------------------------------- sampling

@pytest.mark.parametrize("ptr,idx", [(torch.int32, torch.int32), (torch.int64, torch.int64),
                                     (torch.int32, torch.int64), (torch.int64, torch.int32)])
@pytest.mark.parametrize("fanouts", [[25, 10], [15, 10, 5], [64, 1], [1, 1, 1], [3]])
def test_sampling_parity_hub_graph(mqg, ptr, idx, fanouts):
    rp, ci = hub_graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    deg = np.diff(rp.numpy())
    assert deg.max() > 1000 and (deg <= 3).any()                  # hubs and near-empty rows
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    batch = 193                                                   # ragged: not a multiple of 64
    ctx = mqg.Context(g, batch, fanouts)
    blocks = mqg.Blocks(g, batch, fanouts)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    for b, seeds in enumerate(synth.seed_batches(n, batch, 3, seed=7)):
        got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 55 + b)
        want = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 55 + b)
        assert_blocks_equal(got, want)


@pytest.mark.parametrize("n", [524_288, 524_289, 300])
def test_sampling_on_both_sides_of_the_small_bitmap_limit(mqg, n):
    """Up to 64 bitmap tiles (524,288 nodes) the emit launch counts the tiles before its own itself and
    the relabel launch clears the bitmap; one node more and the counting launch is back.  Two calls in a
    row on one context, so that a bitmap left dirty would show."""
    rp, ci = synth.chung_lu_graph(n, min(1_500_000, 20 * n), max_degree=min(4000, n - 1), seed=5)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts, batch = [10, 10, 5], 700
    ctx = mqg.Context(g, batch, fanouts)
    blocks = mqg.Blocks(g, batch, fanouts)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    for b, seeds in enumerate(synth.seed_batches(n, min(batch, n), 2, seed=11)):
        got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 70 + b)
        want = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 70 + b)
        assert_blocks_equal(got, want)
        assert want[0].num_src >= want[0].num_dst
    # the layer-wise sampler shares the bitmap and the position table: both must be clean again
    lw = mqg.LayerwiseBlocks(g, batch, [200, 200])
    seeds = synth.seed_batches(n, min(batch, n), 1, seed=12)[0]
    mqg.mqg_sample_layerwise(ctx, g, to_dev(seeds), [200, 200], 9, lw)
    torch.cuda.synchronize()
    wl = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), [200, 200], 9)
    hs = lw.host_sizes()
    for l, bl in enumerate(wl):
        assert (hs[l][0], hs[l][1], hs[l][2]) == (bl.num_dst, bl.num_src, bl.nnz)
        assert np.array_equal(lw.src_ids[l][:bl.num_src].cpu().numpy().astype(np.int64), bl.src_ids)
        assert np.array_equal(lw.indices[l][:bl.nnz].cpu().numpy(), bl.indices)


def test_repeated_minimum_selection_path_matches(mqg):
    rp, ci = hub_graph(n=3000, edges=200_000, max_degree=1200)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [20, 7]
    ctx = mqg.Context(g, 64, fanouts)
    ctx.set_option(mqg.MQG_OPT_FORCE_SLOW_SELECT, 1)
    blocks = mqg.Blocks(g, 64, fanouts)
    seeds = synth.seed_batches(rp.numel() - 1, 64, 1, seed=3)[0]
    got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 9)
    want = oracle.sample_blocks(rp.numpy(), ci.numpy(), seeds.numpy(), fanouts, 9)
    assert_blocks_equal(got, want)


@pytest.mark.parametrize("heavy_degree", [None, 64, 500])
def test_workgroup_per_hub_path_matches(mqg, heavy_degree):
    """Rows above the heavy-degree limit are sampled by a whole workgroup; same result."""
    rp, ci = synth.chung_lu_graph(30000, 1_500_000, max_degree=9000, seed=11)
    deg = np.diff(rp.numpy())
    assert deg.max() > 4096                                       # above the default limit of 2048
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [25, 10]
    ctx = mqg.Context(g, 300, fanouts)
    if heavy_degree is not None:
        ctx.set_option(mqg.MQG_OPT_HEAVY_DEGREE, heavy_degree)
    blocks = mqg.Blocks(g, 300, fanouts)
    hubs = torch.from_numpy(np.argsort(-deg)[:100].astype(np.int64))   # the 100 largest hubs as seeds
    rest = synth.seed_batches(rp.numel() - 1, 300, 1, seed=3)[0]
    seeds = torch.unique(torch.cat([hubs, rest]))[:300]
    got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 21)
    want = oracle.sample_blocks(rp.numpy(), ci.numpy(), seeds.numpy(), fanouts, 21)
    assert_blocks_equal(got, want)
    with pytest.raises(mqg.MqgError):
        ctx.set_option(mqg.MQG_OPT_HEAVY_DEGREE, 10)


def test_sampling_edge_cases(mqg):
    # isolated nodes, a node whose neighbours are all destinations, fanout above every degree
    rp = torch.tensor([0, 0, 2, 3, 3, 6], dtype=torch.int64)
    ci = torch.tensor([2, 4, 1, 0, 1, 2], dtype=torch.int64)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [4, 2]
    ctx = mqg.Context(g, 8, fanouts)
    blocks = mqg.Blocks(g, 8, fanouts)
    for seeds in ([0, 1], [4], [3, 0], [0, 1, 2, 3, 4], []):
        s = torch.tensor(seeds, dtype=torch.int64)
        got = hip_sample(mqg, ctx, g, blocks, s, fanouts, 1)
        want = oracle.sample_blocks(rp.numpy(), ci.numpy(), s.numpy(), fanouts, 1)
        assert_blocks_equal(got, want)


def test_eight_layers_until_the_frontier_is_the_whole_graph(mqg):
    """The maximum number of layers; the outer blocks' source lists hold every node of the graph
    (capacity bound min(N, ...)) and most sampled neighbours are already destinations."""
    rp, ci = hub_graph(n=1500, edges=40_000, max_degree=400, seed=8)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [6, 5, 4, 4, 3, 3, 2, 2]
    ctx = mqg.Context(g, 96, fanouts)
    blocks = mqg.Blocks(g, 96, fanouts)
    assert blocks.bounds[0][1] == n                               # capped by the graph size
    for b, seeds in enumerate(synth.seed_batches(n, 96, 2, seed=5)):
        got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 77 + b)
        want = oracle.sample_blocks(rp.numpy(), ci.numpy(), seeds.numpy(), fanouts, 77 + b)
        assert_blocks_equal(got, want)
        reach = want[0].num_src
        assert reach > 0.9 * (np.diff(rp.numpy()) > 0).sum()      # the frontier has saturated
    with pytest.raises(mqg.MqgError):
        mqg.Context(g, 96, [2] * 9)


def test_sampling_is_deterministic_and_context_reusable(mqg):
    rp, ci = hub_graph(n=4000, edges=150_000, max_degree=900)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [10, 10, 5]
    ctx = mqg.Context(g, 128, fanouts)
    blocks = mqg.Blocks(g, 128, fanouts)
    batches = synth.seed_batches(rp.numel() - 1, 128, 2, seed=1)
    a = hip_sample(mqg, ctx, g, blocks, batches[0], fanouts, 5)
    b = hip_sample(mqg, ctx, g, blocks, batches[1], fanouts, 6)     # different batch in between
    c = hip_sample(mqg, ctx, g, blocks, batches[0], fanouts, 5)
    for x, y in zip(a, c):
        for k in ("src_ids", "indptr", "indices"):
            assert np.array_equal(x[k], y[k])
    assert not np.array_equal(a[0]["src_ids"], b[0]["src_ids"])
    # a smaller batch than the context's maximum
    d = hip_sample(mqg, ctx, g, blocks, batches[0][:37], fanouts, 5)
    want = oracle.sample_blocks(rp.numpy(), ci.numpy(), batches[0][:37].numpy(), fanouts, 5)
    assert_blocks_equal(d, want)


def test_four_contexts_on_four_streams_match_one(mqg):
    rp, ci = hub_graph(n=5000, edges=300_000, max_degree=1500)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [15, 10, 5]
    batches = synth.seed_batches(rp.numel() - 1, 256, 4, seed=4)
    ctxs = [mqg.Context(g, 256, fanouts) for _ in range(4)]
    blks = [mqg.Blocks(g, 256, fanouts) for _ in range(4)]
    streams = [torch.cuda.Stream() for _ in range(4)]
    seeds_dev = [to_dev(b) for b in batches]
    torch.cuda.synchronize()
    for i in range(4):
        mqg.mqg_sample_blocks(ctxs[i], g, seeds_dev[i], fanouts, 100 + i, blks[i], stream=streams[i])
    torch.cuda.synchronize()
    for i in range(4):
        want = oracle.sample_blocks(rp.numpy(), ci.numpy(), batches[i].numpy(), fanouts, 100 + i)
        sizes = blks[i].host_sizes()
        for l, wb in enumerate(want):
            nd, ns, nnz, _ = sizes[l]
            assert (nd, ns, nnz) == (wb.num_dst, wb.num_src, wb.nnz)
            assert np.array_equal(blks[i].src_ids[l][:ns].cpu().numpy(), wb.src_ids)
            assert np.array_equal(blks[i].indices[l][:nnz].cpu().numpy(), wb.indices)


# ------------------------------------------------------------------------- cache + gather

@pytest.mark.parametrize("dim,dtype,pct", [(602, torch.float32, 30), (100, torch.float32, 20),
                                           (128, torch.float16, 10), (256, torch.float16, 50),
                                           (64, torch.float32, 0), (7, torch.float16, 100),
                                           (33, torch.float32, 37)])
def test_cache_build_and_gather_parity(mqg, dim, dtype, pct):
    rp, ci = hub_graph(n=9000, edges=300_000, max_degree=2000, seed=dim)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, dim, dtype=dtype, seed=2).pin_memory()
    num_cached = n * pct // 100
    ctx = mqg.Context(g, 256, [8, 4])                            # bounds the id list a gather may classify
    cache = mqg.Cache(g, feats, num_cached)
    mqg.mqg_build_cache(ctx, g, cache)
    torch.cuda.synchronize()
    want = oracle.build_cache(rp.numpy(), num_cached, feats.numpy())
    assert np.array_equal(cache.slot_of.cpu().numpy(), want.slot_of)
    assert np.array_equal(cache.cached_ids[:num_cached].cpu().numpy(), want.cached_ids)
    assert cache.cache_rows[:num_cached].cpu().numpy().tobytes() == want.cache_rows.tobytes()

    rng = np.random.default_rng(5)
    for count in (0, 1, 63, 64, 65, 1500):
        ids_np = rng.permutation(n)[:count].astype(np.int64)
        cap = max(count, 1) + 3
        ids = torch.zeros(cap, dtype=torch.int64, device="cuda")
        ids[:count] = torch.from_numpy(ids_np).cuda()
        num = torch.tensor([count], dtype=torch.int64, device="cuda")
        out = torch.full((cap, dim), 7.0, dtype=dtype, device="cuda")
        stats = torch.zeros(2, dtype=torch.int64, device="cuda")
        mqg.mqg_gather_features(ctx, cache, ids, num, out, stats)
        torch.cuda.synchronize()
        ref, h, m = oracle.gather(ids_np, feats.numpy(), want)
        assert out[:count].cpu().numpy().tobytes() == ref.tobytes()
        assert torch.all(out[count:] == 7.0)
        assert stats.tolist() == [h, m]


def test_gather_result_independent_of_cache_fraction_and_strides(mqg):
    rp, ci = hub_graph(n=5000, edges=120_000, max_degree=800)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    dim = 50
    feats = synth.node_features(n, dim, dtype=torch.float32, seed=3).pin_memory()
    ctx = mqg.Context(g, 256, [10])
    ids_np = np.random.default_rng(1).permutation(n)[:2000].astype(np.int64)
    ids = torch.from_numpy(ids_np).cuda()
    num = torch.tensor([2000], dtype=torch.int64, device="cuda")
    ref = feats.numpy()[ids_np]
    for num_cached, cache_stride, out_stride in [(None, None, 50), (0, 52, 50), (n // 5, 64, 56), (n, 50, 51)]:
        cache = mqg.Cache(g, feats, num_cached, cache_stride)
        if num_cached is not None:
            mqg.mqg_build_cache(ctx, g, cache)
        buf = torch.zeros((2000, out_stride), dtype=torch.float32, device="cuda")
        out = buf[:, :dim]
        mqg.mqg_gather_features(ctx, cache, ids, num, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), ref)                 # padding columns are unspecified
    # int32 ids take the same path
    cache = mqg.Cache(g, feats, n // 5)
    mqg.mqg_build_cache(ctx, g, cache)
    out = torch.zeros((2000, dim), dtype=torch.float32, device="cuda")
    mqg.mqg_gather_features(ctx, cache, ids.to(torch.int32), num, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), ref)


@pytest.mark.parametrize("dim,dtype", [(602, torch.float32), (50, torch.float32), (100, torch.float16), (1, torch.float16)])
def test_gather_copies_whole_lines_between_line_aligned_rows(mqg, dim, dtype):
    """Cache rows and output rows on 64-byte boundaries: the HBM-to-HBM copy moves whole 64-byte
    lines; the columns of a row are the same, rows past the count stay untouched."""
    rp, ci = hub_graph(n=6000, edges=150_000, max_degree=900, seed=4)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    elt = 2 if dtype == torch.float16 else 4
    stride = (dim * elt + 63) // 64 * 64 // elt
    feats = synth.node_features(n, dim, dtype=dtype, seed=6).pin_memory()
    ctx = mqg.Context(g, 256, [10])
    want = oracle.build_cache(rp.numpy(), n // 2, feats.numpy())
    for feats_side in (feats, feats.cuda()):                      # misses from host, or every row from HBM
        cache = mqg.Cache(g, feats_side, n // 2, cache_stride=stride)
        mqg.mqg_build_cache(ctx, g, cache)
        for count in (0, 1, 130, 1999):
            ids_np = np.random.default_rng(count).permutation(n)[:count].astype(np.int64)
            cap = count + 2
            ids = torch.zeros(cap, dtype=torch.int64, device="cuda")
            ids[:count] = torch.from_numpy(ids_np).cuda()
            num = torch.tensor([count], dtype=torch.int64, device="cuda")
            buf = torch.full((cap, stride), 7.0, dtype=dtype, device="cuda")
            stats = torch.zeros(2, dtype=torch.int64, device="cuda")
            mqg.mqg_gather_features(ctx, cache, ids, num, buf[:, :dim], stats)
            torch.cuda.synchronize()
            ref, h, m = oracle.gather(ids_np, feats.numpy(), want)
            assert buf[:count, :dim].contiguous().cpu().numpy().tobytes() == ref.tobytes()
            assert torch.all(buf[count:] == 7.0)
            assert stats.tolist() == [h, m]


@pytest.mark.parametrize("dim,dtype", [(602, torch.float32), (100, torch.float32), (128, torch.float16), (3, torch.float16)])
def test_gather_ids_outside_the_graph_are_skipped_and_show_in_the_stats(mqg, dim, dtype):
    """An id outside [0, num_nodes) is never used as an index: its output row keeps what it held,
    it counts in neither stat, and nothing beyond the buffers is written - through the cache, without
    a cache (features in HBM and in host memory), and through the entry point without a context."""
    rp, ci = hub_graph(n=6000, edges=150_000, max_degree=900, seed=4)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, dim, dtype=dtype, seed=6).pin_memory()
    ctx = mqg.Context(g, 256, [10])
    count = 2500
    rng = np.random.default_rng(8)
    ids_np = rng.permutation(n)[:count].astype(np.int64)
    bad_pos = rng.permutation(count)[:37]
    bad_vals = np.array([n, n + 1, -1, -7, 2 ** 31 - 1, 2 ** 40, -2 ** 40, n + 10 ** 6], dtype=np.int64)
    good = np.ones(count, dtype=bool)
    good[bad_pos] = False
    want_cache = oracle.build_cache(rp.numpy(), n // 3, feats.numpy())
    ref, h, m = oracle.gather(ids_np[good], feats.numpy(), want_cache)
    for idx_dtype in (torch.int64, torch.int32):
        bv = bad_vals if idx_dtype == torch.int64 else bad_vals[np.abs(bad_vals) < 2 ** 31]
        ids_bad = ids_np.copy()
        ids_bad[bad_pos] = bv[np.arange(len(bad_pos)) % len(bv)]
        ids = torch.from_numpy(ids_bad).to(idx_dtype).cuda()
        num = torch.tensor([count], dtype=torch.int64, device="cuda")
        cached = mqg.Cache(g, feats, n // 3)
        mqg.mqg_build_cache(ctx, g, cached)
        for what, cache in (("cache", cached), ("direct-host", mqg.Cache(g, feats, None)),
                            ("direct-hbm", mqg.Cache(g, feats.cuda(), None))):
            for static in (False, True):
                buf = torch.full((count + 5, dim), 7.0, dtype=dtype, device="cuda")
                stats = torch.full((2,), -1, dtype=torch.int64, device="cuda")
                if static:
                    mqg.mqg_gather_features_static(cache, ids, num, buf[:count], stats)
                else:
                    mqg.mqg_gather_features(ctx, cache, ids, num, buf[:count], stats)
                torch.cuda.synchronize()
                got = buf.cpu().numpy()
                assert got[:count][good].tobytes() == ref.tobytes(), (what, static)
                assert np.all(got[:count][~good] == 7.0) and np.all(got[count:] == 7.0), (what, static)
                assert stats.tolist() == ([h, m] if what == "cache" else [0, int(good.sum())]), (what, static)
        # a clean call afterwards counts from zero again
        stats = torch.zeros(2, dtype=torch.int64, device="cuda")
        out = torch.zeros((count, dim), dtype=dtype, device="cuda")
        mqg.mqg_gather_features(ctx, mqg.Cache(g, feats, None), torch.from_numpy(ids_np).to(idx_dtype).cuda(), num, out, stats)
        torch.cuda.synchronize()
        assert stats.tolist() == [0, count]


@pytest.mark.parametrize("dim,dtype", [(602, torch.float32), (100, torch.float32), (128, torch.float16)])
def test_gather_in_two_halves_equals_the_whole(mqg, dim, dtype):
    """mqg_gather_features_cached on one stream, mqg_gather_features_missed on another, ordered by an
    event: same rows and stats as the single call and as the oracle - several gathers in a row on one
    context, also without a cache."""
    rp, ci = hub_graph(n=9000, edges=200_000, max_degree=1200, seed=6)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, dim, dtype=dtype, seed=9).pin_memory()
    elt = feats.element_size()
    stride = (dim * elt + 63) // 64 * 64 // elt
    ctx = mqg.Context(g, 512, [12])
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for num_cached in (n // 4, 0, None):
        cache = mqg.Cache(g, feats, num_cached, cache_stride=stride if num_cached is not None else None)
        want = None
        if num_cached is not None:
            mqg.mqg_build_cache(ctx, g, cache)
            want = oracle.build_cache(rp.numpy(), num_cached, feats.numpy())
        torch.cuda.synchronize()
        for count in (4000, 0, 777, 6000):
            ids_np = np.random.default_rng(count).permutation(n)[:count].astype(np.int64)
            cap = count + 1
            ids = torch.zeros(cap, dtype=torch.int64, device="cuda")
            ids[:count] = torch.from_numpy(ids_np).cuda()
            num = torch.tensor([count], dtype=torch.int64, device="cuda")
            whole = torch.full((cap, stride), 7.0, dtype=dtype, device="cuda")
            st_whole = torch.zeros(2, dtype=torch.int64, device="cuda")
            mqg.mqg_gather_features(ctx, cache, ids, num, whole[:, :dim], st_whole)
            torch.cuda.synchronize()
            halves = torch.full((cap, stride), 7.0, dtype=dtype, device="cuda")
            st_halves = torch.zeros(2, dtype=torch.int64, device="cuda")
            ev = torch.cuda.Event()
            mqg.mqg_gather_features_cached(ctx, cache, ids, num, halves[:, :dim], st_halves, stream=s1)
            ev.record(s1)
            s2.wait_event(ev)
            mqg.mqg_gather_features_missed(ctx, cache, ids, num, halves[:, :dim], st_halves, stream=s2)
            torch.cuda.synchronize()
            ref, h, m = oracle.gather(ids_np, feats.numpy(), want)
            assert halves[:count, :dim].contiguous().cpu().numpy().tobytes() == ref.tobytes(), (num_cached, count)
            assert whole[:count, :dim].contiguous().cpu().numpy().tobytes() == ref.tobytes(), (num_cached, count)
            assert torch.all(halves[count:] == 7.0)
            assert st_halves.tolist() == st_whole.tolist() == [h, m], (num_cached, count)


def test_cache_ties_and_many_equal_degrees(mqg):
    # ring: every degree equal -> cache is the lowest ids; then a star on top
    n = 5000
    src = torch.arange(n)
    und = torch.stack([src, (src + 1) % n])
    both = torch.cat([und, und.flip(0)], 1)
    key = torch.unique(both[0] * n + both[1])
    rows, cols = key // n, key % n
    rp = torch.zeros(n + 1, dtype=torch.int64)
    rp[1:] = torch.cumsum(torch.bincount(rows, minlength=n), 0)
    g = mqg.Graph(to_dev(rp), to_dev(cols.contiguous()))
    feats = synth.node_features(n, 4, seed=1).pin_memory()
    ctx = mqg.Context(g, 8, [2])
    cache = mqg.Cache(g, feats, 777)
    mqg.mqg_build_cache(ctx, g, cache)
    torch.cuda.synchronize()
    want = oracle.build_cache(rp.numpy(), 777, feats.numpy())
    assert want.cached_ids.tolist() == list(range(777))
    assert np.array_equal(cache.cached_ids.cpu().numpy(), want.cached_ids)
    assert np.array_equal(cache.slot_of.cpu().numpy(), want.slot_of)


# ------------------------------------------------------------------------- aggregate

@pytest.mark.parametrize("dim,dtype", [(64, np.float32), (100, np.float32), (602, np.float32),
                                       (128, np.float16), (256, np.float16), (7, np.float32),
                                       (9, np.float16), (1030, np.float32)])
def test_mean_aggregate_parity_random_blocks(mqg, dim, dtype):
    rng = np.random.default_rng(dim)
    nd, ns = 777, 3000
    counts = rng.integers(0, 26, nd)
    counts[::50] = 0                                             # empty rows
    indptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    indices = rng.integers(0, ns, indptr[-1]).astype(np.int32)
    x = rng.standard_normal((ns, dim)).astype(dtype)
    ref = oracle.mean_aggregate(indptr, indices, x)
    # a bare block descriptor: only indptr / indices / sizes matter to the aggregation
    rp = torch.tensor([0, 0], dtype=torch.int64)
    g = mqg.Graph(to_dev(rp), torch.zeros(1, dtype=torch.int64, device="cuda"))
    ctx = mqg.Context(g, 1, [1])
    blocks = mqg.Blocks(g, 1, [1])
    ip, ix = to_dev(torch.from_numpy(indptr)), to_dev(torch.from_numpy(indices))
    sizes = torch.tensor([nd, ns, int(indptr[-1]), 0], dtype=torch.int64, device="cuda")
    blocks.c[0] = mqg.CBlock(nd, ns, int(indptr[-1]), None, ip.data_ptr(), ix.data_ptr(), sizes.data_ptr())
    blocks.bounds[0] = (nd, ns, int(indptr[-1]))
    xd = to_dev(torch.from_numpy(x))
    out = torch.full((nd + 2, dim), 5.0, dtype=xd.dtype, device="cuda")
    mqg.mqg_sage_mean_aggregate(ctx, blocks, 0, xd, out)
    torch.cuda.synchronize()
    got = out[:nd].cpu().numpy()
    ok, worst = agg_tolerance_ok(got, ref, float(np.abs(x.astype(np.float64)).mean()), TOL[dtype])
    assert ok, worst
    assert torch.all(out[nd:] == 5.0)
    assert np.all(got[counts == 0] == 0)
    # closed form: constant features give the constant back exactly
    const = torch.full((ns, dim), 1.5, dtype=xd.dtype, device="cuda")
    mqg.mqg_sage_mean_aggregate(ctx, blocks, 0, const, out)
    torch.cuda.synchronize()
    got = out[:nd].cpu().numpy()
    assert np.all(got[counts > 0] == 1.5)


# ------------------------------------------------------------------------- scaled and full-size workloads

@pytest.mark.parametrize("name,factor,batches", [("medium", 0.04, 2), ("large", 0.02, 2), ("stress", 0.01, 1)])
def test_scaled_workloads_whole_path(mqg, name, factor, batches):
    w = synth.scaled(synth.WORKLOADS[name], factor)
    if name == "stress":
        w = dataclasses.replace(w, batch=1024)
    rp, ci = synth.build_graph(w, seed=0)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, w.dim, dtype=w.feat_dtype, seed=1).pin_memory()
    ctx = mqg.Context(g, w.batch, w.fanouts)
    blocks = mqg.Blocks(g, w.batch, w.fanouts)
    cache = mqg.Cache(g, feats, n * w.cache_pct // 100)
    mqg.mqg_build_cache(ctx, g, cache)
    ocache = oracle.build_cache(rp.numpy(), n * w.cache_pct // 100, feats.numpy())
    assert np.array_equal(cache.slot_of.cpu().numpy(), ocache.slot_of)
    npdt = np.float16 if w.feat_dtype == torch.float16 else np.float32
    for b, seeds in enumerate(synth.seed_batches(n, w.batch, batches, seed=2)):
        got = hip_sample(mqg, ctx, g, blocks, seeds, w.fanouts, 7 + b)
        want = oracle.sample_blocks(rp.numpy(), ci.numpy(), seeds.numpy(), w.fanouts, 7 + b)
        assert_blocks_equal(got, want)
        cap = blocks.bounds[0][1]
        x0 = torch.zeros((cap, w.dim), dtype=w.feat_dtype, device="cuda")
        stats = torch.zeros(2, dtype=torch.int64, device="cuda")
        mqg.mqg_gather_features(ctx, cache, blocks.src_ids[0], blocks.sizes[0, 1:2], x0, stats)
        torch.cuda.synchronize()
        ref_rows, h, m = oracle.gather(want[0].src_ids, feats.numpy(), ocache)
        assert x0[:want[0].num_src].cpu().numpy().tobytes() == ref_rows.tobytes()
        assert stats.tolist() == [h, m]
        run_aggregate_chain(mqg, ctx, blocks, x0, want, ref_rows, npdt)


# ------------------------------------------------------------------------- error handling

def test_bad_seeds_are_flagged_on_the_device_not_dereferenced(mqg):
    rp, ci = hub_graph(n=3000, edges=40_000, max_degree=300)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [4, 3]
    ctx = mqg.Context(g, 8, fanouts)
    blocks = mqg.Blocks(g, 8, fanouts)

    def flags_of(seeds):
        mqg.mqg_sample_blocks(ctx, g, to_dev(torch.tensor(seeds, dtype=torch.int64)), fanouts, 5, blocks)
        torch.cuda.synchronize()
        return blocks.host_sizes()

    sz = flags_of([5, n + 7, 9, -3])                              # two ids outside the graph
    assert sz[1][3] & 1 and sz[0][3] == 0
    assert blocks.src_ids[1][:4].tolist() == [5, 0, 9, 0]         # replaced by node 0 (and now repeated)
    assert sz[1][3] & 2
    sz = flags_of([5, 9, 5])                                      # a repeated id
    assert sz[1][3] == 2
    # the context is clean afterwards: a good batch is bit-exact and unflagged
    got = hip_sample(mqg, ctx, g, blocks, torch.tensor([1, 2, 3, 4]), fanouts, 6)
    want = oracle.sample_blocks(rp.numpy(), ci.numpy(), np.array([1, 2, 3, 4]), fanouts, 6)
    assert_blocks_equal(got, want)


def test_host_side_errors(mqg):
    rp, ci = hub_graph(n=2000, edges=20_000, max_degree=200)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    with pytest.raises(mqg.MqgError) as e:
        mqg.Context(g, 16, [65])
    assert e.value.code == mqg.MQG_ERR_UNSUPPORTED
    with pytest.raises(mqg.MqgError):
        mqg.Context(g, 16, [])
    ctx = mqg.Context(g, 16, [5, 5])
    blocks = mqg.Blocks(g, 16, [5, 5])
    seeds = to_dev(torch.arange(32, dtype=torch.int64))
    with pytest.raises(mqg.MqgError) as e:                       # more seeds than the context allows
        mqg.mqg_sample_blocks(ctx, g, seeds, [5, 5], 0, blocks)
    assert e.value.code == mqg.MQG_ERR_CAPACITY
    with pytest.raises(mqg.MqgError) as e:                       # fanout above the context's
        mqg.mqg_sample_blocks(ctx, g, seeds[:16], [5, 6], 0, blocks)
    assert e.value.code == mqg.MQG_ERR_CAPACITY
    with pytest.raises(mqg.MqgError) as e:                       # layer count mismatch
        mqg.mqg_sample_blocks(ctx, g, seeds[:16], [5], 0, blocks)
    assert e.value.code == mqg.MQG_ERR_INVALID_ARG
    small = mqg.Blocks(g, 8, [5, 5])                             # buffers below the bound
    with pytest.raises(mqg.MqgError) as e:
        mqg.mqg_sample_blocks(ctx, g, seeds[:16], [5, 5], 0, small)
    assert e.value.code == mqg.MQG_ERR_CAPACITY and "cap_" in str(e.value)
    # the context still works after refused calls
    got = hip_sample(mqg, ctx, g, blocks, torch.arange(16, dtype=torch.int64), [5, 5], 3)
    want = oracle.sample_blocks(rp.numpy(), ci.numpy(), np.arange(16), [5, 5], 3)
    assert_blocks_equal(got, want)
