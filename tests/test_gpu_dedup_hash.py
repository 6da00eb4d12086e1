"""Sampling with the hash-table dedup (MQG_OPT_DEDUP_HASH) versus the oracle, through the C ABI:
the blocks must be the same, bit for bit, as with the node-indexed tables."""
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


@pytest.mark.parametrize("ptr,idx", [(torch.int32, torch.int32), (torch.int64, torch.int64)])
@pytest.mark.parametrize("fanouts", [[25, 10], [15, 10, 5], [64, 1], [1, 1, 1], [3]])
def test_hash_dedup_parity_hub_graph(mqg, ptr, idx, fanouts):
    rp, ci = hub_graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    batch = 193
    ctx = mqg.Context(g, batch, fanouts)
    ctx.set_option(mqg.MQG_OPT_DEDUP_HASH, 1)
    blocks = mqg.Blocks(g, batch, fanouts)
    for b, seeds in enumerate(synth.seed_batches(n, batch, 3, seed=7)):
        got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 55 + b)
        want = oracle.sample_blocks(rp.numpy(), ci.numpy(), seeds.numpy(), fanouts, 55 + b)
        assert_blocks_equal(got, want)


def test_hash_dedup_small_graph_where_frontier_saturates(mqg):
    """The frontier reaches every node: the table holds the whole graph."""
    rp, ci = synth.chung_lu_graph(700, 30_000, max_degree=300, seed=2)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [20, 20, 20]
    ctx = mqg.Context(g, 256, fanouts)
    ctx.set_option(mqg.MQG_OPT_DEDUP_HASH, 1)
    blocks = mqg.Blocks(g, 256, fanouts)
    seeds = synth.seed_batches(700, 256, 1, seed=9)[0]
    got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 3)
    want = oracle.sample_blocks(rp.numpy(), ci.numpy(), seeds.numpy(), fanouts, 3)
    assert_blocks_equal(got, want)
    assert got[0]["num_src"] > 600


def test_switching_between_the_two_dedup_paths_on_one_context(mqg):
    rp, ci = hub_graph(n=4000, edges=150_000, max_degree=900)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [10, 10, 5]
    ctx = mqg.Context(g, 128, fanouts)
    blocks = mqg.Blocks(g, 128, fanouts)
    batches = synth.seed_batches(rp.numel() - 1, 128, 4, seed=1)
    for i, mode in enumerate([1, 0, 1, 0]):
        ctx.set_option(mqg.MQG_OPT_DEDUP_HASH, mode)
        seeds = batches[i] if i != 2 else batches[i][:37]           # also a smaller batch
        got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 5 + i)
        want = oracle.sample_blocks(rp.numpy(), ci.numpy(), seeds.numpy(), fanouts, 5 + i)
        assert_blocks_equal(got, want)


def test_hash_dedup_edge_cases_and_flags(mqg):
    rp = torch.tensor([0, 0, 2, 3, 3, 6], dtype=torch.int64)
    ci = torch.tensor([2, 4, 1, 0, 1, 2], dtype=torch.int64)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [4, 2]
    ctx = mqg.Context(g, 8, fanouts)
    ctx.set_option(mqg.MQG_OPT_DEDUP_HASH, 1)
    blocks = mqg.Blocks(g, 8, fanouts)
    for seeds in ([0, 1], [4], [3, 0], [0, 1, 2, 3, 4], []):
        s = torch.tensor(seeds, dtype=torch.int64)
        got = hip_sample(mqg, ctx, g, blocks, s, fanouts, 1)
        want = oracle.sample_blocks(rp.numpy(), ci.numpy(), s.numpy(), fanouts, 1)
        assert_blocks_equal(got, want)

    def sizes_of(seeds):
        mqg.mqg_sample_blocks(ctx, g, to_dev(torch.tensor(seeds, dtype=torch.int64)), fanouts, 5, blocks)
        torch.cuda.synchronize()
        return blocks.host_sizes()

    sz = sizes_of([2, 11, 4, -3])                                 # two ids outside the graph -> node 0, twice
    assert sz[1][3] == 3 and sz[0][3] == 0
    assert blocks.src_ids[1][:4].tolist() == [2, 0, 4, 0]
    sz = sizes_of([2, 4, 2])
    assert sz[1][3] == 2
    got = hip_sample(mqg, ctx, g, blocks, torch.tensor([1, 2, 3]), fanouts, 6)
    want = oracle.sample_blocks(rp.numpy(), ci.numpy(), np.array([1, 2, 3]), fanouts, 6)
    assert_blocks_equal(got, want)


@pytest.mark.parametrize("name", ["medium", "large"])
def test_hash_dedup_full_size_three_in_flight(mqg, name):
    """At the benchmark's sizes and launch configuration: three contexts on three streams."""
    w = synth.WORKLOADS[name]
    rp, ci = synth.build_graph(w, seed=0, device="cuda")
    n = rp.numel() - 1
    g = mqg.Graph(rp, ci)
    fanouts = list(w.fanouts)
    ctxs = [mqg.Context(g, w.batch, fanouts) for _ in range(3)]
    for c in ctxs:
        c.set_option(mqg.MQG_OPT_DEDUP_HASH, 1)
    blks = [mqg.Blocks(g, w.batch, fanouts) for _ in range(3)]
    streams = [torch.cuda.Stream() for _ in range(3)]
    batches = synth.seed_batches(n, w.batch, 3, seed=12)
    seeds_dev = [b.to(g.idx_dtype).cuda() for b in batches]
    torch.cuda.synchronize()
    for rep in range(2):                                          # the second round reuses the cleared tables
        for i in range(3):
            mqg.mqg_sample_blocks(ctxs[i], g, seeds_dev[i], fanouts, 40 + i, blks[i], stream=streams[i])
    torch.cuda.synchronize()
    rp_np, ci_np = rp.cpu().numpy(), ci.cpu().numpy()
    for i in range(3):
        want = oracle.sample_blocks(rp_np, ci_np, batches[i].numpy(), fanouts, 40 + i)
        sizes = blks[i].host_sizes()
        for l, wb in enumerate(want):
            nd, ns, nnz, flags = sizes[l]
            assert (nd, ns, nnz, flags) == (wb.num_dst, wb.num_src, wb.nnz, 0)
            assert np.array_equal(blks[i].src_ids[l][:ns].cpu().numpy(), wb.src_ids)
            assert np.array_equal(blks[i].indptr[l][:nd + 1].cpu().numpy(), wb.indptr)
            assert np.array_equal(blks[i].indices[l][:nnz].cpu().numpy(), wb.indices)
