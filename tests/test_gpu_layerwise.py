"""Layer-wise (LADIES) sampling on the GPU versus the oracle, through the C ABI.

Which nodes are drawn, the source lists, indptr and indices must be identical (integer masses and
correctly rounded double keys on both sides).  Edge weights are floating point: relative
tolerance 1e-6 (computed in double on both sides and rounded to float once on the GPU; the sums
over the candidates and over a row are taken in another order than the oracle's)."""
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


def hub_graph(n=20000, edges=400_000, max_degree=3000, ptr=torch.int64, idx=torch.int64, seed=1):
    rp, ci = synth.chung_lu_graph(n, edges, max_degree=max_degree, seed=seed)
    return rp.to(ptr), ci.to(idx)


def run_layerwise(mqg, ctx, g, blocks, seeds_cpu, sizes, rng_seed, normalise=True, method=0):
    seeds = to_dev(seeds_cpu.to(g.idx_dtype))
    mqg.mqg_sample_layerwise(ctx, g, seeds, sizes, rng_seed, blocks, normalise=normalise, method=method)
    torch.cuda.synchronize()
    hs = blocks.host_sizes()
    out = []
    for l in range(len(sizes)):
        nd, ns, nnz, flags = hs[l]
        out.append(dict(num_dst=nd, num_src=ns, nnz=nnz, flags=flags,
                        src_ids=blocks.src_ids[l][:ns].cpu().numpy().astype(np.int64),
                        indptr=blocks.indptr[l][:nd + 1].cpu().numpy().astype(np.int64),
                        indices=blocks.indices[l][:nnz].cpu().numpy(),
                        edge_w=blocks.edge_w[l][:nnz].cpu().numpy()))
    return out


def assert_same(got, want, flags=0):
    assert len(got) == len(want)
    for l, (a, b) in enumerate(zip(got, want)):
        assert (a["num_dst"], a["num_src"], a["nnz"], a["flags"]) == (b.num_dst, b.num_src, b.nnz, flags), l
        assert np.array_equal(a["src_ids"], b.src_ids), l
        assert np.array_equal(a["indptr"], b.indptr), l
        assert np.array_equal(a["indices"], b.indices), l
        assert np.allclose(a["edge_w"], b.edge_w, rtol=1e-6, atol=0), l


@pytest.mark.parametrize("ptr,idx", [(torch.int32, torch.int32), (torch.int64, torch.int64), (torch.int64, torch.int32)])
@pytest.mark.parametrize("sizes", [[64, 128], [512, 512], [100, 50, 30], [7]])
@pytest.mark.parametrize("normalise", [True, False])
def test_layerwise_parity_hub_graph(mqg, ptr, idx, sizes, normalise):
    rp, ci = hub_graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    batch = 193
    ctx = mqg.Context(g, batch, [2] * len(sizes))
    blocks = mqg.LayerwiseBlocks(g, batch, sizes)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    for b, seeds in enumerate(synth.seed_batches(n, batch, 2, seed=7)):
        got = run_layerwise(mqg, ctx, g, blocks, seeds, sizes, 55 + b, normalise)
        want = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 55 + b, normalise=normalise)
        assert_same(got, want)
        if normalise:
            for a in got:
                sums = np.add.reduceat(np.concatenate([a["edge_w"], [0.0]]), np.minimum(a["indptr"][:-1], a["nnz"]))
                nonempty = np.diff(a["indptr"]) > 0
                assert np.allclose(sums[nonempty], 1.0, rtol=1e-5)


@pytest.mark.parametrize("ptr,idx", [(torch.int32, torch.int32), (torch.int64, torch.int64)])
@pytest.mark.parametrize("sizes", [[64, 128], [512, 512], [100, 50, 30]])
def test_fastgcn_parity_and_alternation_with_ladies(mqg, ptr, idx, sizes):
    rp, ci = hub_graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    batch = 193
    ctx = mqg.Context(g, batch, [2] * len(sizes))
    blocks = mqg.LayerwiseBlocks(g, batch, sizes)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    batches = synth.seed_batches(n, batch, 2, seed=7)
    prev = None
    for b, seeds in enumerate(batches):
        for normalise in (True, False):
            got = run_layerwise(mqg, ctx, g, blocks, seeds, sizes, 55, normalise, method=mqg.MQG_LAYERWISE_FASTGCN)
            want = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 55, normalise=normalise, fastgcn=True)
            assert_same(got, want)
        if prev is not None:                                      # same sampling seed: the same nodes for another batch
            for l in range(len(sizes)):
                assert np.array_equal(prev[l]["src_ids"], got[l]["src_ids"])
        prev = got
        # LADIES on the same context in between: its masses and candidate lists are separate
        got = run_layerwise(mqg, ctx, g, blocks, seeds, sizes, 56)
        assert_same(got, oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 56))


@pytest.mark.parametrize("ptr,idx", [(torch.int32, torch.int32), (torch.int64, torch.int64)])
@pytest.mark.parametrize("sizes", [[64, 128], [512, 512], [100, 50, 30], [3000]])
@pytest.mark.parametrize("fastgcn,debias", [(False, False), (True, False), (False, True), (True, True)])
def test_flat_variants_parity(mqg, ptr, idx, sizes, fastgcn, debias):
    """The "+flat" variants (Eq. 10: drawn in proportion to the column norm, squared tickets in the
    race) alone and combined with FastGCN's masses and the debiased coefficients."""
    rp, ci = hub_graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    batch = 193
    ctx = mqg.Context(g, batch, [2] * len(sizes))
    blocks = mqg.LayerwiseBlocks(g, batch, sizes)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    method = (mqg.MQG_LAYERWISE_FLAT | (mqg.MQG_LAYERWISE_FASTGCN if fastgcn else 0) | (mqg.MQG_LAYERWISE_DEBIAS if debias else 0))
    for b, seeds in enumerate(synth.seed_batches(n, batch, 2, seed=7)):
        for normalise in (True, False):
            got = run_layerwise(mqg, ctx, g, blocks, seeds, sizes, 91 + b, normalise, method=method)
            want = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 91 + b, normalise=normalise, fastgcn=fastgcn,
                                        debias=debias, flat=True)
            assert_same(got, want)
    # not the same draw as without the flag
    plain = run_layerwise(mqg, ctx, g, blocks, seeds, sizes, 91, True, method=method & ~mqg.MQG_LAYERWISE_FLAT)
    flat = run_layerwise(mqg, ctx, g, blocks, seeds, sizes, 91, True, method=method)
    if plain[-1]["num_src"] == sizes[-1] and sizes[-1] < 1000:   # a real draw (not every candidate taken)
        assert not np.array_equal(plain[-1]["src_ids"], flat[-1]["src_ids"])
    with pytest.raises(mqg.MqgError):
        mqg.mqg_sample_layerwise(ctx, g, to_dev(seeds.to(g.idx_dtype)), sizes, 1, blocks, method=8)


@pytest.mark.parametrize("ptr,idx", [(torch.int32, torch.int32), (torch.int64, torch.int64)])
@pytest.mark.parametrize("sizes", [[64, 128], [512, 512], [100, 50, 30], [3000]])
@pytest.mark.parametrize("fastgcn", [False, True])
def test_debiased_variants_parity(mqg, ptr, idx, sizes, fastgcn):
    rp, ci = hub_graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    batch = 193
    ctx = mqg.Context(g, batch, [2] * len(sizes))
    blocks = mqg.LayerwiseBlocks(g, batch, sizes)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    seeds = synth.seed_batches(n, batch, 1, seed=7)[0]
    method = mqg.MQG_LAYERWISE_DEBIAS | (mqg.MQG_LAYERWISE_FASTGCN if fastgcn else 0)
    for normalise in (False, True):
        got = run_layerwise(mqg, ctx, g, blocks, seeds, sizes, 91, normalise, method=method)
        want = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 91, normalise=normalise, fastgcn=fastgcn, debias=True)
        assert_same(got, want)
    plain = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 91, normalise=False, fastgcn=fastgcn)
    want = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 91, normalise=False, fastgcn=fastgcn, debias=True)
    assert not np.allclose(plain[-1].edge_w, want[-1].edge_w, rtol=1e-5)      # the coefficients do differ from 1 / (s p)


@pytest.mark.parametrize("sizes", [[64, 128], [512, 512], [100, 50, 30], [30000]])
def test_layerwise_candidate_paths_give_the_same_blocks(mqg, sizes):
    """The three ways to a layer's candidates - a key slot per node, a list read off the masses, a
    list from bits set slot by slot (the last two are what graphs above 1 M / 8 M nodes take) -
    against the oracle, alternating on one context, plain and debiased."""
    rp, ci = hub_graph()
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    batch = 193
    ctx = mqg.Context(g, batch, [2] * len(sizes))
    blocks = mqg.LayerwiseBlocks(g, batch, sizes)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    seeds = synth.seed_batches(n, batch, 3, seed=17)
    for b, how in enumerate([3, 1, 2, 3, 2, 1, 0]):
        ctx.set_option(mqg.MQG_OPT_LAYERWISE_CANDIDATES, how)
        debias = b % 2 == 1
        got = run_layerwise(mqg, ctx, g, blocks, seeds[b % 3], sizes, 90 + b, method=mqg.MQG_LAYERWISE_DEBIAS if debias else 0)
        want = oracle.ladies_blocks(rp_np, ci_np, seeds[b % 3].numpy(), sizes, 90 + b, debias=debias)
        assert_same(got, want)
    with pytest.raises(mqg.MqgError):
        ctx.set_option(mqg.MQG_OPT_LAYERWISE_CANDIDATES, 4)


def test_layerwise_small_graph_all_candidates_and_degenerate_inputs(mqg):
    rp = torch.tensor([0, 0, 2, 3, 3, 6], dtype=torch.int64)      # nodes 0 and 3 have no neighbours
    ci = torch.tensor([2, 4, 1, 0, 1, 2], dtype=torch.int64)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    ctx = mqg.Context(g, 8, [2, 2])
    for sizes in ([4, 4], [1, 1], [100, 2]):
        blocks = mqg.LayerwiseBlocks(g, 8, sizes)
        for seeds in ([0], [1, 3], [4, 2, 1], [0, 1, 2, 3, 4], []):
            s = torch.tensor(seeds, dtype=torch.int64)
            for normalise in (True, False):
                got = run_layerwise(mqg, ctx, g, blocks, s, sizes, 3, normalise)
                want = oracle.ladies_blocks(rp.numpy(), ci.numpy(), s.numpy(), sizes, 3, normalise=normalise)
                assert_same(got, want)
                got = run_layerwise(mqg, ctx, g, blocks, s, sizes, 3, normalise, method=mqg.MQG_LAYERWISE_FASTGCN)
                want = oracle.ladies_blocks(rp.numpy(), ci.numpy(), s.numpy(), sizes, 3, normalise=normalise, fastgcn=True)
                assert_same(got, want)
                got = run_layerwise(mqg, ctx, g, blocks, s, sizes, 3, normalise, method=mqg.MQG_LAYERWISE_DEBIAS)
                want = oracle.ladies_blocks(rp.numpy(), ci.numpy(), s.numpy(), sizes, 3, normalise=normalise, debias=True)
                assert_same(got, want)
    # an id outside the graph is replaced by node 0 and flagged on the innermost block
    blocks = mqg.LayerwiseBlocks(g, 8, [4, 4])
    got = run_layerwise(mqg, ctx, g, blocks, torch.tensor([2, 9, -1]), [4, 4], 5)
    assert got[1]["flags"] == 1 and got[0]["flags"] == 0
    want = oracle.ladies_blocks(rp.numpy(), ci.numpy(), np.array([2, 0, 0]), [4, 4], 5)
    assert np.array_equal(got[1]["src_ids"], want[1].src_ids)
    got = run_layerwise(mqg, ctx, g, blocks, torch.tensor([2, 4]), [4, 4], 5)      # the flag does not stick
    assert got[1]["flags"] == 0


def test_layerwise_edge_capacity_overflow_is_flagged_not_written(mqg):
    rp, ci = hub_graph(n=3000, edges=200_000, max_degree=1200)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    sizes = [256, 256]
    ctx = mqg.Context(g, 64, [2, 2])
    blocks = mqg.LayerwiseBlocks(g, 64, sizes, nnz_per_row=2)     # far too few edge slots
    guard = [t.clone() for t in blocks.indices]
    seeds = synth.seed_batches(3000, 64, 1, seed=3)[0]
    got = run_layerwise(mqg, ctx, g, blocks, seeds, sizes, 9)
    want = oracle.ladies_blocks(rp.numpy(), ci.numpy(), seeds.numpy(), sizes, 9)
    for l in (0, 1):
        assert want[l].nnz > blocks.bounds[l][2]
        assert got[l]["flags"] == 4 and got[l]["nnz"] == blocks.bounds[l][2]
        assert np.array_equal(got[l]["src_ids"], want[l].src_ids)            # the draw itself is unaffected
        assert np.array_equal(got[l]["indices"], want[l].indices[:got[l]["nnz"]])
    del guard


def test_layerwise_leaves_the_context_clean_and_feeds_the_weighted_aggregation(mqg):
    rp, ci = hub_graph(n=5000, edges=300_000, max_degree=1500)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [10, 5]
    sizes = [300, 200]
    ctx = mqg.Context(g, 128, fanouts)
    nw_blocks = mqg.Blocks(g, 128, fanouts)
    lw_blocks = mqg.LayerwiseBlocks(g, 128, sizes)
    seeds = synth.seed_batches(n, 128, 1, seed=4)[0]
    rp_np, ci_np = rp.numpy(), ci.numpy()
    want_nw = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 8)
    want_lw = oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 8)
    for _ in range(2):                                            # alternate the two samplers on one context
        assert_same(run_layerwise(mqg, ctx, g, lw_blocks, seeds, sizes, 8), want_lw)
        assert_blocks_equal(hip_sample(mqg, ctx, g, nw_blocks, seeds, fanouts, 8), want_nw)
    got = run_layerwise(mqg, ctx, g, lw_blocks, seeds, sizes, 8)
    # H_{l+1} = block_l weighted sums of H_l, chained from the outermost block
    dim = 40
    rng = np.random.default_rng(2)
    x = rng.standard_normal((want_lw[0].num_src, dim)).astype(np.float32)
    xd = torch.zeros((lw_blocks.bounds[0][1], dim), device="cuda")
    xd[:x.shape[0]] = torch.from_numpy(x).cuda()
    for l in range(2):
        b = want_lw[l]
        ref = oracle.weighted_aggregate(b.indptr, b.indices, b.edge_w, None, x)
        out = torch.zeros((lw_blocks.bounds[l][0], dim), device="cuda")
        mqg.mqg_weighted_aggregate(ctx, lw_blocks, l, lw_blocks.edge_w[l], None, xd, out)
        torch.cuda.synchronize()
        o = out[:b.num_dst].cpu().numpy()
        mass = np.abs(x.astype(np.float64)).mean()
        assert np.all(np.abs(o - ref) <= 1e-5 * np.maximum(np.abs(ref), mass)), l
        x, xd = ref, out
    assert got[1]["num_dst"] == 128


def test_layerwise_full_size_medium(mqg):
    """The paper's setting for layer-wise samplers (512 nodes per layer, two layers) on the
    "medium" graph with 1,024 seeds."""
    w = synth.WORKLOADS["medium"]
    rp, ci = synth.build_graph(w, seed=0, device="cuda")
    n = rp.numel() - 1
    g = mqg.Graph(rp, ci)
    sizes = [512, 512]
    ctx = mqg.Context(g, w.batch, [2, 2])
    blocks = mqg.LayerwiseBlocks(g, w.batch, sizes)
    seeds = synth.seed_batches(n, w.batch, 2, seed=12)
    rp_np, ci_np = rp.cpu().numpy(), ci.cpu().numpy()
    for i in range(2):
        got = run_layerwise(mqg, ctx, g, blocks, seeds[i], sizes, 40 + i)
        want = oracle.ladies_blocks(rp_np, ci_np, seeds[i].numpy(), sizes, 40 + i)
        assert_same(got, want)
        assert want[0].num_src == 512 and want[1].nnz > 1024


@pytest.mark.parametrize("n,k,distinct", [(5000, 512, 7), (5000, 512, 2 ** 40), (70000, 3000, 300), (300, 299, 5),
                                          (300, 300, 5), (300, 1000, 5), (64, 1, 1), (1, 1, 1), (100000, 1, 2 ** 62),
                                          (5000, 1234, 1), (3000, 2999, 2), (1025, 1024, 1), (1024, 1, 1)])
def test_selection_step_with_many_equal_keys(mqg, n, k, distinct):
    """The radix select against a full sort, on keys drawn from a small set so that the threshold
    key is shared by many candidates of which only some fit."""
    rp = torch.tensor([0, 0], dtype=torch.int64)
    g = mqg.Graph(to_dev(rp), torch.zeros(1, dtype=torch.int64, device="cuda"))
    ctx = mqg.Context(g, 1, [1])
    rng = np.random.default_rng(n + k)
    vals = rng.integers(0, 2 ** 63, size=min(distinct, 4 * n), dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, size=min(distinct, 4 * n), dtype=np.uint64)
    keys = vals[rng.integers(0, len(vals), n)]                   # the top bit is set in about half of them
    got = mqg.mqg_select_smallest_keys(ctx, torch.from_numpy(keys.view(np.int64)).cuda(), k)
    torch.cuda.synchronize()
    order = np.lexsort((np.arange(n), keys))
    want = np.zeros(n, dtype=bool)
    want[order[:min(k, n)]] = True
    assert np.array_equal(got.cpu().numpy(), want)


@pytest.mark.parametrize("low_bits", [1, 5, 12, 13, 14, 26, 27, 39, 40, 52, 53, 64])
def test_selection_step_when_only_the_low_bits_differ(mqg, low_bits):
    """Keys that share everything above their lowest `low_bits` bits: the select has to carry its
    prefix through the passes whose digit is the same for every key (the widths straddle the digit
    boundaries at bits 13, 26, 39 and 52)."""
    n, k = 20000, 777
    rp = torch.tensor([0, 0], dtype=torch.int64)
    g = mqg.Graph(to_dev(rp), torch.zeros(1, dtype=torch.int64, device="cuda"))
    ctx = mqg.Context(g, 1, [1])
    rng = np.random.default_rng(low_bits)
    high = np.uint64(0x3FE5A5A5A5A5A5A5) if low_bits < 64 else np.uint64(0)
    mask = np.uint64((1 << low_bits) - 1) if low_bits < 64 else np.uint64(2 ** 64 - 1)
    low = rng.integers(0, 2 ** 63, size=n, dtype=np.uint64) * np.uint64(2) + rng.integers(0, 2, size=n, dtype=np.uint64)
    keys = (high & ~mask) | (low & mask)
    got = mqg.mqg_select_smallest_keys(ctx, torch.from_numpy(keys.view(np.int64)).cuda(), k)
    torch.cuda.synchronize()
    order = np.lexsort((np.arange(n), keys))
    want = np.zeros(n, dtype=bool)
    want[order[:k]] = True
    assert np.array_equal(got.cpu().numpy(), want)


def test_samplers_do_not_need_sorted_adjacency_rows(mqg):
    """Rows in arbitrary order (the generators emit ascending rows; nothing in the library may rely
    on it): node-wise, cache-prioritised and layer-wise sampling against the oracle."""
    rp, ci = hub_graph(n=6000, edges=200_000, max_degree=1500)
    n = rp.numel() - 1
    rng = np.random.default_rng(0)
    ci_np = ci.numpy().copy()
    rp_np = rp.numpy()
    for v in range(n):
        rng.shuffle(ci_np[rp_np[v]:rp_np[v + 1]])
    assert not np.all(np.diff(ci_np[rp_np[100]:rp_np[101]]) > 0) or rp_np[101] - rp_np[100] < 3
    g = mqg.Graph(to_dev(rp), to_dev(torch.from_numpy(ci_np)))
    fanouts, sizes = [12, 6], [200, 150]
    ctx = mqg.Context(g, 100, fanouts)
    blocks = mqg.Blocks(g, 100, fanouts)
    lw = mqg.LayerwiseBlocks(g, 100, sizes)
    feats = synth.node_features(n, 4, seed=2).pin_memory()
    cache = mqg.Cache(g, feats, n // 6)
    mqg.mqg_build_cache(ctx, g, cache)
    torch.cuda.synchronize()
    slot_of = cache.slot_of.cpu().numpy()
    seeds = synth.seed_batches(n, 100, 1, seed=8)[0]
    assert_blocks_equal(hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 4),
                        oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 4))
    ctx.set_sampling_priority(cache)
    assert_blocks_equal(hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 4),
                        oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 4, prio_slot_of=slot_of))
    ctx.set_sampling_priority(None)
    for method, fg in ((mqg.MQG_LAYERWISE_LADIES, False), (mqg.MQG_LAYERWISE_FASTGCN, True)):
        assert_same(run_layerwise(mqg, ctx, g, lw, seeds, sizes, 4, method=method),
                    oracle.ladies_blocks(rp_np, ci_np, seeds.numpy(), sizes, 4, fastgcn=fg))
