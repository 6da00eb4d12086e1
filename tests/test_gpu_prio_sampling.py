"""Cache-prioritised neighbour sampling on the GPU versus the oracle, through the C ABI: bit-exact
blocks, on and off, after a cache rebuild, with both dedup paths, and at the "medium" workload's
full size in the benchmark's launch configuration."""
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
@pytest.mark.parametrize("fanouts", [[25, 10], [15, 10, 5], [64, 1], [3]])
@pytest.mark.parametrize("pct", [1, 30])
def test_prioritised_sampling_parity(mqg, ptr, idx, fanouts, pct):
    rp, ci = hub_graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, 4, seed=2).pin_memory()
    batch = 193
    ctx = mqg.Context(g, batch, fanouts)
    blocks = mqg.Blocks(g, batch, fanouts)
    cache = mqg.Cache(g, feats, n * pct // 100)
    mqg.mqg_build_cache(ctx, g, cache)
    ctx.set_sampling_priority(cache)
    slot_of = cache.slot_of.cpu().numpy()
    want_cache = oracle.build_cache(rp.numpy(), n * pct // 100)
    assert np.array_equal(slot_of, want_cache.slot_of)
    rp_np, ci_np = rp.numpy(), ci.numpy()
    for b, seeds in enumerate(synth.seed_batches(n, batch, 2, seed=7)):
        got = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 55 + b)
        want = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 55 + b, prio_slot_of=slot_of)
        assert_blocks_equal(got, want)
    plain = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 56)
    if pct == 30 and fanouts[0] > 1:
        assert not np.array_equal(plain[0].src_ids, want[0].src_ids)       # the priority changes the draw


def test_prioritised_unconditional_selection_and_switching(mqg):
    rp, ci = hub_graph(n=3000, edges=200_000, max_degree=1200)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, 4, seed=2).pin_memory()
    fanouts = [20, 7]
    ctx = mqg.Context(g, 64, fanouts)
    blocks = mqg.Blocks(g, 64, fanouts)
    cache = mqg.Cache(g, feats, n // 8)
    mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_DEGREE_SAMPLED, seed=3)
    torch.cuda.synchronize()
    slot_of = cache.slot_of.cpu().numpy()
    seeds = synth.seed_batches(n, 64, 1, seed=3)[0]
    rp_np, ci_np = rp.numpy(), ci.numpy()
    want_prio = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 9, prio_slot_of=slot_of)
    want_plain = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 9)
    ctx.set_sampling_priority(cache)
    assert_blocks_equal(hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 9), want_prio)
    ctx.set_option(mqg.MQG_OPT_FORCE_SLOW_SELECT, 1)              # every row through the repeated-minimum path
    assert_blocks_equal(hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 9), want_prio)
    ctx.set_option(mqg.MQG_OPT_FORCE_SLOW_SELECT, 0)
    ctx.set_option(mqg.MQG_OPT_HEAVY_DEGREE, 64)                  # every long row through the workgroup-per-row path
    assert_blocks_equal(hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 9), want_prio)
    ctx.set_option(mqg.MQG_OPT_HEAVY_DEGREE, 2048)
    ctx.set_option(mqg.MQG_OPT_DEDUP_HASH, 1)                     # with the hash-table dedup
    assert_blocks_equal(hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 9), want_prio)
    ctx.set_option(mqg.MQG_OPT_DEDUP_HASH, 0)
    ctx.set_sampling_priority(None)                               # off again: the uniform draw
    assert_blocks_equal(hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 9), want_plain)
    # a rebuilt cache (another epoch's draw) and the priority set again
    mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_DEGREE_SAMPLED, seed=4)
    ctx.set_sampling_priority(cache)
    torch.cuda.synchronize()
    slot_of2 = cache.slot_of.cpu().numpy()
    assert not np.array_equal(slot_of, slot_of2)
    want2 = oracle.sample_blocks(rp_np, ci_np, seeds.numpy(), fanouts, 9, prio_slot_of=slot_of2)
    assert_blocks_equal(hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 9), want2)
    # argument errors
    rp2, ci2 = hub_graph(n=500, edges=3000, max_degree=50)
    g2 = mqg.Graph(to_dev(rp2), to_dev(ci2))
    other = mqg.Cache(g2, synth.node_features(500, 4, seed=2).pin_memory(), 10)
    with pytest.raises(mqg.MqgError):
        ctx.set_sampling_priority(other)


def test_prioritised_sampling_full_size_medium_three_in_flight(mqg):
    w = synth.WORKLOADS["medium"]
    rp, ci = synth.build_graph(w, seed=0, device="cuda")
    n = rp.numel() - 1
    g = mqg.Graph(rp, ci)
    fanouts = list(w.fanouts)
    feats = torch.zeros((n, 8), dtype=torch.float32).pin_memory()
    ctxs = [mqg.Context(g, w.batch, fanouts) for _ in range(3)]
    cache = mqg.Cache(g, feats, n * w.cache_pct // 100)
    mqg.mqg_build_cache(ctxs[0], g, cache)
    torch.cuda.synchronize()
    for c in ctxs:
        c.set_sampling_priority(cache)
    blks = [mqg.Blocks(g, w.batch, fanouts) for _ in range(3)]
    streams = [torch.cuda.Stream() for _ in range(3)]
    batches = synth.seed_batches(n, w.batch, 3, seed=12)
    seeds_dev = [b.to(g.idx_dtype).cuda() for b in batches]
    torch.cuda.synchronize()
    for i in range(3):
        mqg.mqg_sample_blocks(ctxs[i], g, seeds_dev[i], fanouts, 40 + i, blks[i], stream=streams[i])
    torch.cuda.synchronize()
    rp_np, ci_np = rp.cpu().numpy(), ci.cpu().numpy()
    slot_of = cache.slot_of.cpu().numpy()
    for i in range(3):
        want = oracle.sample_blocks(rp_np, ci_np, batches[i].numpy(), fanouts, 40 + i, prio_slot_of=slot_of)
        sizes = blks[i].host_sizes()
        for l, wb in enumerate(want):
            nd, ns, nnz, flags = sizes[l]
            assert (nd, ns, nnz, flags) == (wb.num_dst, wb.num_src, wb.nnz, 0)
            assert np.array_equal(blks[i].src_ids[l][:ns].cpu().numpy(), wb.src_ids)
            assert np.array_equal(blks[i].indptr[l][:nd + 1].cpu().numpy(), wb.indptr)
            assert np.array_equal(blks[i].indices[l][:nnz].cpu().numpy(), wb.indices)
    plain = oracle.sample_blocks(rp_np, ci_np, batches[0].numpy(), fanouts, 40)
    want0 = oracle.sample_blocks(rp_np, ci_np, batches[0].numpy(), fanouts, 40, prio_slot_of=slot_of)
    unc = lambda b: int((slot_of[b[0].src_ids] < 0).sum())
    assert unc(want0) < 0.5 * unc(plain)                          # what the priority is for
