"""Seeded random configurations of the sampler through the C ABI against the oracle: graph size and
skew, index types, number of layers, fanouts, batch size, hub threshold, dedup path and cache
priority all drawn at random, so that combinations no hand-written case lists are exercised
(bit-exact blocks, gathered rows byte for byte)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_04707_amd import synth
from gpu_util import assert_blocks_equal, hip_sample, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mqg():
    from paper_2601_04707_amd import mqg as m
    assert torch.cuda.is_available()
    return m


def draw_config(rng):
    n = int(rng.choice([3, 40, 700, 2500, 6000]))
    mean_deg = float(rng.choice([1.5, 6, 30, 120]))
    edges = max(4, int(n * mean_deg))
    max_degree = int(min(n - 1, rng.choice([8, 70, 300, 2500])))
    L = int(rng.integers(1, 5))
    fanouts = [int(rng.choice([1, 2, 5, 10, 15, 25, 40, 64])) for _ in range(L)]
    batch = int(min(n, rng.choice([1, 7, 64, 65, 200])))
    return dict(n=n, edges=edges, max_degree=max(1, max_degree), fanouts=fanouts, batch=batch,
                ptr=rng.choice([torch.int32, torch.int64]), idx=rng.choice([torch.int32, torch.int64]),
                heavy=rng.choice([None, 64, 100, 500]), hash_dedup=bool(rng.integers(0, 2)),
                prio_pct=rng.choice([None, None, 5, 50]), graph_seed=int(rng.integers(0, 1 << 30)),
                rng_seed=int(rng.integers(0, 1 << 62)))


@pytest.mark.parametrize("case", range(48))
def test_random_configuration(mqg, case):
    rng = np.random.default_rng(9000 + case)
    c = draw_config(rng)
    rp, ci = synth.chung_lu_graph(c["n"], c["edges"], max_degree=c["max_degree"], seed=c["graph_seed"],
                                  ptr_dtype=c["ptr"], idx_dtype=c["idx"])
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    ctx = mqg.Context(g, c["batch"], c["fanouts"])
    blocks = mqg.Blocks(g, c["batch"], c["fanouts"])
    if c["heavy"] is not None:
        ctx.set_option(mqg.MQG_OPT_HEAVY_DEGREE, int(c["heavy"]))
    if c["hash_dedup"]:
        ctx.set_option(mqg.MQG_OPT_DEDUP_HASH, 1)
    dim = int(rng.choice([1, 8, 50, 150]))
    feats = synth.node_features(n, dim, seed=3).pin_memory()
    num_cached = 0 if c["prio_pct"] is None else n * int(c["prio_pct"]) // 100
    cache = mqg.Cache(g, feats, num_cached)
    mqg.mqg_build_cache(ctx, g, cache)
    slot_of = None
    if c["prio_pct"] is not None:
        ctx.set_sampling_priority(cache)
        slot_of = oracle.build_cache(rp.numpy(), num_cached).slot_of
    rp_np, ci_np = rp.numpy(), ci.numpy()
    for b, seeds in enumerate(synth.seed_batches(n, c["batch"], 2, seed=case)):
        got = hip_sample(mqg, ctx, g, blocks, seeds, c["fanouts"], c["rng_seed"] + b)
        want = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), c["fanouts"], c["rng_seed"] + b, prio_slot_of=slot_of)
        assert_blocks_equal(got, want)
        x0 = torch.zeros((blocks.bounds[0][1], dim), dtype=torch.float32, device="cuda")
        stats = torch.zeros(2, dtype=torch.int64, device="cuda")
        mqg.mqg_gather_features(ctx, cache, blocks.src_ids[0], blocks.sizes[0, 1:2], x0, stats)
        torch.cuda.synchronize()
        ns = want[0].num_src
        assert x0[:ns].cpu().numpy().tobytes() == feats.numpy()[want[0].src_ids].tobytes()
        assert int(stats.sum()) == ns


@pytest.mark.parametrize("case", range(24))
def test_random_layerwise_configuration(mqg, case):
    """The layer-wise sampler (LADIES / FastGCN, with and without flat probabilities, debiasing and row normalisation) on
    random graph shapes, layer sizes and batch sizes, through a random one of its three ways to a
    layer's candidates: drawn nodes and block structure identical, edge weights to 1e-6."""
    rng = np.random.default_rng(7000 + case)
    n = int(rng.choice([5, 60, 900, 4000]))
    edges = max(4, int(n * float(rng.choice([2, 10, 60]))))
    max_degree = max(1, int(min(n - 1, rng.choice([6, 80, 1500]))))
    ptr, idx = rng.choice([torch.int32, torch.int64]), rng.choice([torch.int32, torch.int64])
    rp, ci = synth.chung_lu_graph(n, edges, max_degree=max_degree, seed=int(rng.integers(0, 1 << 30)),
                                  ptr_dtype=ptr, idx_dtype=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    L = int(rng.integers(1, 4))
    sizes = [int(rng.choice([1, 3, 40, 300, 2000])) for _ in range(L)]
    batch = int(min(n, rng.choice([1, 9, 64, 130])))
    fastgcn, debias, normalise, flat = (bool(rng.integers(0, 2)) for _ in range(4))
    method = ((mqg.MQG_LAYERWISE_FASTGCN if fastgcn else mqg.MQG_LAYERWISE_LADIES) | (mqg.MQG_LAYERWISE_DEBIAS if debias else 0) |
              (mqg.MQG_LAYERWISE_FLAT if flat else 0))
    ctx = mqg.Context(g, batch, [2] * L)
    ctx.set_option(mqg.MQG_OPT_LAYERWISE_CANDIDATES, int(rng.choice([0, 1, 2, 3])))   # the paths of larger graphs too
    blocks = mqg.LayerwiseBlocks(g, batch, sizes)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    for b, seeds in enumerate(synth.seed_batches(n, batch, 2, seed=case)):
        rng_seed = int(rng.integers(0, 1 << 62))
        mqg.mqg_sample_layerwise(ctx, g, to_dev(seeds.to(g.idx_dtype)), sizes, rng_seed, blocks, normalise=normalise, method=method)
        torch.cuda.synchronize()
        want = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, rng_seed, normalise=normalise, fastgcn=fastgcn, debias=debias, flat=flat)
        hs = blocks.host_sizes()
        for l, w in enumerate(want):
            nd, ns, nnz, flags = hs[l]
            assert (nd, ns, nnz, flags) == (w.num_dst, w.num_src, w.nnz, 0), (l, hs[l])
            assert np.array_equal(blocks.src_ids[l][:ns].cpu().numpy().astype(np.int64), w.src_ids), l
            assert np.array_equal(blocks.indptr[l][:nd + 1].cpu().numpy().astype(np.int64), w.indptr), l
            assert np.array_equal(blocks.indices[l][:nnz].cpu().numpy(), w.indices), l
            assert np.allclose(blocks.edge_w[l][:nnz].cpu().numpy(), w.edge_w, rtol=1e-6, atol=0), l


def directed_graph(n, mean_out, seed, idx=torch.int64):
    """A directed simple graph in CSR (row v = in-neighbours of v), skewed in-degrees, rows unsorted."""
    rng = np.random.default_rng(seed)
    m = int(n * mean_out)
    dst = np.minimum((rng.pareto(1.3, m) * 3).astype(np.int64), n - 1)      # a few nodes receive most edges
    dst = rng.permutation(n)[dst]
    src = rng.integers(0, n, m)
    keep = src != dst
    pairs = np.unique(np.stack([dst[keep], src[keep]], 1), axis=0)
    pairs = pairs[rng.permutation(len(pairs))]
    order = np.argsort(pairs[:, 0], kind="stable")                          # rows grouped, neighbours in random order
    pairs = pairs[order]
    rp = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rp, pairs[:, 0] + 1, 1)
    rp = np.cumsum(rp)
    return torch.from_numpy(rp), torch.from_numpy(pairs[:, 1].copy()).to(idx)


@pytest.mark.parametrize("seed", [1, 2])
def test_directed_graph_all_paths(mqg, seed):
    """The synthetic workloads are symmetrised; nothing in the library may rely on that.  A directed
    graph with unsorted rows through node-wise sampling, the layer-wise sampler, the random-walk
    cache scores and the Eq. 1-3 weights, each against the oracle."""
    rp, ci = directed_graph(3000, 25, seed)
    n = rp.numel() - 1
    rp_np, ci_np = rp.numpy(), ci.numpy()
    indeg = np.diff(rp_np)
    outdeg = np.bincount(ci_np, minlength=n)
    assert not np.array_equal(indeg, outdeg) and indeg.max() > 300
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [12, 6]
    batch = 150
    ctx = mqg.Context(g, batch, fanouts)
    blocks = mqg.Blocks(g, batch, fanouts)
    seeds = synth.seed_batches(n, batch, 1, seed=seed)[0]
    got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 31)
    want = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 31)
    assert_blocks_equal(got, want)

    # Eq. 1-3 weights of the sampled blocks
    for l, wb in enumerate(want):
        ew = torch.zeros(blocks.bounds[l][2], dtype=torch.float32, device="cuda")
        sw = torch.zeros(blocks.bounds[l][0], dtype=torch.float32, device="cuda")
        mqg.mqg_gcn_edge_weights(ctx, g, blocks, l, ew, sw)
        torch.cuda.synchronize()
        ref_e, ref_s = oracle.gcn_edge_weights(rp_np, wb.src_ids, wb.indptr, wb.indices)
        assert np.allclose(ew[:wb.nnz].cpu().numpy(), ref_e, rtol=1e-6, atol=0)
        assert np.allclose(sw[:wb.num_dst].cpu().numpy(), ref_s, rtol=1e-6, atol=0)

    # random-walk cache scores: bit-identical doubles
    train = torch.randperm(n, generator=torch.Generator().manual_seed(4))[:60]
    feats = synth.node_features(n, 6, seed=3).pin_memory()
    cache = mqg.Cache(g, feats, n // 10)
    scores = torch.zeros(n, dtype=torch.float64, device="cuda")
    mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_RANDOM_WALK, train_ids=to_dev(train), step_fanouts=[6, 12],
                           scores_out=scores)
    torch.cuda.synchronize()
    want_scores = oracle.random_walk_scores(rp_np, ci_np, train.numpy(), [6, 12])
    assert np.array_equal(scores.cpu().numpy(), want_scores)
    wc = oracle.build_cache_by_score(want_scores, n // 10, feats.numpy())
    assert np.array_equal(cache.slot_of.cpu().numpy(), wc.slot_of)
    mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_RANDOM_WALK, train_ids=to_dev(train), step_fanouts=[6, 12],
                           scores_out=scores, walk_form=mqg.MQG_WALK_PRINTED)
    torch.cuda.synchronize()
    assert np.array_equal(scores.cpu().numpy(), oracle.random_walk_scores(rp_np, ci_np, train.numpy(), [6, 12], oracle.WALK_PRINTED))

    # layer-wise sampler
    sizes = [200, 100]
    lb = mqg.LayerwiseBlocks(g, batch, sizes)
    for method, kw in [(mqg.MQG_LAYERWISE_LADIES, {}), (mqg.MQG_LAYERWISE_FASTGCN | mqg.MQG_LAYERWISE_DEBIAS, dict(fastgcn=True, debias=True))]:
        mqg.mqg_sample_layerwise(ctx, g, to_dev(seeds), sizes, 77, lb, normalise=True, method=method)
        torch.cuda.synchronize()
        wl = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 77, normalise=True, **kw)
        hs = lb.host_sizes()
        for l, w in enumerate(wl):
            nd, ns, nnz, flags = hs[l]
            assert (nd, ns, nnz, flags) == (w.num_dst, w.num_src, w.nnz, 0)
            assert np.array_equal(lb.src_ids[l][:ns].cpu().numpy().astype(np.int64), w.src_ids)
            assert np.array_equal(lb.indices[l][:nnz].cpu().numpy(), w.indices)
            assert np.allclose(lb.edge_w[l][:nnz].cpu().numpy(), w.edge_w, rtol=1e-6, atol=0)
