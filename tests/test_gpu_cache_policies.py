"""The paper's own cache policies on the GPU versus the oracle: membership drawn in proportion to
in-degree (Eq. 13) and short-random-walk scores (Eq. 14-15).  Bit-exact, scores included."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_04707_amd import synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mqg():
    from paper_2601_04707_amd import mqg as m
    assert torch.cuda.is_available()
    return m


def graph(n=20000, edges=400_000, max_degree=3000, seed=1, ptr=torch.int64, idx=torch.int64):
    return synth.chung_lu_graph(n, edges, max_degree=max_degree, seed=seed, ptr_dtype=ptr, idx_dtype=idx)


@pytest.mark.parametrize("ptr,idx", [(torch.int64, torch.int64), (torch.int32, torch.int32)])
def test_degree_sampled_cache_parity_and_redraw(mqg, ptr, idx):
    rp, ci = graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    deg = np.diff(rp.numpy())
    assert deg.max() > 1000 and (deg == 0).any()
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, 12, seed=2).pin_memory()
    ctx = mqg.Context(g, 8, [2])
    seen = []
    for num_cached, seed in [(n // 100, 0), (n // 100, 1), (n // 3, 7), (n, 3), (0, 5)]:
        cache = mqg.Cache(g, feats, num_cached)
        mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_DEGREE_SAMPLED, seed=seed)
        torch.cuda.synchronize()
        want = oracle.build_cache_sampled(rp.numpy(), num_cached, seed, feats.numpy())
        assert np.array_equal(cache.cached_ids[:num_cached].cpu().numpy(), want.cached_ids)
        assert np.array_equal(cache.slot_of.cpu().numpy(), want.slot_of)
        assert cache.cache_rows[:num_cached].cpu().numpy().tobytes() == want.cache_rows.tobytes()
        seen.append(want.cached_ids)
    assert not np.array_equal(seen[0], seen[1])                   # a new epoch seed redraws the cache
    # drawn in proportion to degree: the cached 1 % hold far more than 1 % of the edge endpoints
    assert deg[seen[0]].sum() / deg.sum() > 0.05
    # gathers through a sampled cache give the same rows
    cache = mqg.Cache(g, feats, n // 10)
    mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_DEGREE_SAMPLED, seed=11)
    ids = torch.randperm(n)[:8 + 2 * 8].to(torch.int64).cuda()
    out = torch.zeros((ids.numel(), 12), device="cuda")
    mqg.mqg_gather_features(ctx, cache, ids, torch.tensor([ids.numel()], device="cuda"), out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), feats.numpy()[ids.cpu().numpy()])


@pytest.mark.parametrize("ptr,idx", [(torch.int64, torch.int64), (torch.int32, torch.int64)])
@pytest.mark.parametrize("fanouts", [[5], [15, 10, 5], [10 ** 6, 10 ** 6], []])
def test_random_walk_cache_parity(mqg, ptr, idx, fanouts):
    rp, ci = graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, 6, seed=3).pin_memory()
    ctx = mqg.Context(g, 8, [2])
    train = torch.randperm(n, generator=torch.Generator().manual_seed(4))[: n // 100].to(idx)
    num_cached = n // 20
    cache = mqg.Cache(g, feats, num_cached)
    scores = torch.zeros(n, dtype=torch.float64, device="cuda")
    mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_RANDOM_WALK, train_ids=to_dev(train), step_fanouts=fanouts,
                           scores_out=scores)
    torch.cuda.synchronize()
    want_scores = oracle.random_walk_scores(rp.numpy(), ci.numpy(), train.numpy(), fanouts)
    got_scores = scores.cpu().numpy()
    assert np.array_equal(got_scores, want_scores), float(np.abs(got_scores - want_scores).max())
    want = oracle.build_cache_by_score(want_scores, num_cached, feats.numpy())
    assert np.array_equal(cache.cached_ids[:num_cached].cpu().numpy(), want.cached_ids)
    assert np.array_equal(cache.slot_of.cpu().numpy(), want.slot_of)
    assert cache.cache_rows[:num_cached].cpu().numpy().tobytes() == want.cache_rows.tobytes()
    if fanouts:
        # the scores favour what a sampler starting at the training set reaches
        reach = np.zeros(n, dtype=bool)
        reach[train.numpy()] = True
        assert reach[want.cached_ids[: len(train) // 2]].mean() > 0.05 or want_scores[want.cached_ids[0]] > 1.0 / len(train)


@pytest.mark.parametrize("ptr,idx", [(torch.int64, torch.int64), (torch.int32, torch.int32)])
def test_cache_drawn_from_random_walk_scores_parity(mqg, ptr, idx):
    rp, ci = graph(ptr=ptr, idx=idx)
    n = rp.numel() - 1
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(n, 6, seed=3).pin_memory()
    ctx = mqg.Context(g, 8, [2])
    train = torch.randperm(n, generator=torch.Generator().manual_seed(4))[: n // 100].to(idx)
    fanouts = [10, 5]
    want_scores = oracle.random_walk_scores(rp.numpy(), ci.numpy(), train.numpy(), fanouts)
    assert (want_scores == 0).any() and (want_scores > 0).sum() > n // 2
    seen = []
    for num_cached, seed in [(n // 100, 0), (n // 100, 1), (n // 5, 2), (n, 3)]:   # n: past the nodes with a positive score
        cache = mqg.Cache(g, feats, num_cached)
        scores = torch.zeros(n, dtype=torch.float64, device="cuda")
        mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_RANDOM_WALK_SAMPLED, seed=seed, train_ids=to_dev(train),
                               step_fanouts=fanouts, scores_out=scores)
        torch.cuda.synchronize()
        assert np.array_equal(scores.cpu().numpy(), want_scores)
        want = oracle.build_cache_drawn_by_score(want_scores, num_cached, seed, feats.numpy())
        assert np.array_equal(cache.cached_ids[:num_cached].cpu().numpy(), want.cached_ids)
        assert np.array_equal(cache.slot_of.cpu().numpy(), want.slot_of)
        assert cache.cache_rows[:num_cached].cpu().numpy().tobytes() == want.cache_rows.tobytes()
        seen.append(want.cached_ids)
    assert not np.array_equal(seen[0], seen[1])                   # another seed, another draw
    assert want_scores[seen[0]].mean() > 3 * want_scores.mean()   # drawn towards high scores
    assert (want_scores[seen[0]] > 0).all()


def test_policy_argument_errors(mqg):
    rp, ci = graph(n=2000, edges=20_000, max_degree=200)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    feats = synth.node_features(2000, 4, seed=3).pin_memory()
    ctx = mqg.Context(g, 8, [2])
    cache = mqg.Cache(g, feats, 10)
    with pytest.raises(mqg.MqgError):
        mqg.mqg_build_cache_ex(ctx, g, cache, 9)
    with pytest.raises(mqg.MqgError):
        mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_RANDOM_WALK, train_ids=None, step_fanouts=[0])
    with pytest.raises(mqg.MqgError):
        mqg.mqg_build_cache_ex(ctx, g, cache, mqg.MQG_CACHE_RANDOM_WALK, step_fanouts=[5] * 9)
    # top degree through the extended call equals the plain call
    a, b = mqg.Cache(g, feats, 100), mqg.Cache(g, feats, 100)
    mqg.mqg_build_cache(ctx, g, a)
    mqg.mqg_build_cache_ex(ctx, g, b, mqg.MQG_CACHE_TOP_DEGREE)
    torch.cuda.synchronize()
    assert torch.equal(a.slot_of, b.slot_of) and torch.equal(a.cached_ids, b.cached_ids)
