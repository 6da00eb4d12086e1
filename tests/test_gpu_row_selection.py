"""The per-row selection of the sampling kernels (binary radix select on wavefront ballots) fed with
crafted candidates through the C ABI: the chosen set must be the first k of a plain sort by
(late flag, key, slot), also when many keys are exactly equal - a case that real 64-bit sampling
keys never produce, so the block parity tests cannot reach it."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    from paper_2601_04707_amd import mqg as m
    assert torch.cuda.is_available()
    rp = torch.tensor([0, 1, 2], dtype=torch.int64, device="cuda")
    ci = torch.tensor([1, 0], dtype=torch.int64, device="cuda")
    g = m.Graph(rp, ci)
    return m, m.Context(g, 2, [1])


def expected(keys_u64, slots, late, k, prioritised):
    order = sorted(range(len(keys_u64)), key=lambda c: ((late[c] if prioritised else 0), int(keys_u64[c]), int(slots[c]), c))
    chosen = np.zeros(len(keys_u64), dtype=bool)
    chosen[order[:k]] = True
    return chosen


def run(m, ctx, keys_u64, slots, late, k, prioritised, ordered):
    words = (slots.astype(np.uint32) | (late.astype(np.uint32) << 31)).view(np.int32)
    got = m.mqg_select_row_candidates(ctx, torch.from_numpy(keys_u64.view(np.int64)).cuda(), torch.from_numpy(words).cuda(),
                                      k, prioritised=prioritised, ordered=ordered)
    torch.cuda.synchronize()
    return got.cpu().numpy()


def key_sets(rng, n):
    full = rng.integers(0, 2**63, n, dtype=np.int64).astype(np.uint64) * np.uint64(2) + rng.integers(0, 2, n).astype(np.uint64)
    yield "random", full
    yield "all equal", np.full(n, 0x0123456789ABCDEF, dtype=np.uint64)
    yield "three values", rng.choice(np.array([0, 2**63, 2**64 - 1], dtype=np.uint64), n)
    yield "low bits only", rng.integers(0, 4, n).astype(np.uint64)
    yield "high word ties", (rng.integers(0, 3, n).astype(np.uint64) << np.uint64(32)) | rng.integers(0, 5, n).astype(np.uint64)
    yield "extremes", np.where(rng.random(n) < 0.5, np.uint64(0), np.uint64(2**64 - 1)).astype(np.uint64)


@pytest.mark.parametrize("n", [1, 2, 63, 64, 65, 128, 129, 200, 256])
@pytest.mark.parametrize("prioritised", [False, True])
def test_selection_in_slot_order_with_ties(env, n, prioritised):
    """Candidates stored in ascending slot order (the one-wavefront-per-row path)."""
    m, ctx = env
    rng = np.random.default_rng(n * 2 + int(prioritised))
    slots = np.sort(rng.choice(5000, n, replace=False)).astype(np.int64)
    for name, keys in key_sets(rng, n):
        late = (rng.random(n) < 0.4).astype(np.int64)
        for k in sorted({1, min(n, 2), min(n, 25), min(n, 64), n}):
            got = run(m, ctx, keys, slots, late, k, prioritised, ordered=True)
            want = expected(keys, slots, late, k, prioritised)
            assert np.array_equal(got, want), (name, n, k)


@pytest.mark.parametrize("n", [1, 64, 65, 130, 256])
@pytest.mark.parametrize("prioritised", [False, True])
def test_selection_of_unordered_candidates_with_ties(env, n, prioritised):
    """Candidates in arrival order (the hub path): equal keys are resolved by slot value."""
    m, ctx = env
    rng = np.random.default_rng(1000 + n * 2 + int(prioritised))
    slots = rng.permutation(40000)[:n].astype(np.int64)
    for name, keys in key_sets(rng, n):
        late = (rng.random(n) < 0.4).astype(np.int64)
        for k in sorted({1, min(n, 10), min(n, 64), n}):
            got = run(m, ctx, keys, slots, late, k, prioritised, ordered=False)
            want = expected(keys, slots, late, k, prioritised)
            assert np.array_equal(got, want), (name, n, k)


def test_selection_argument_errors(env):
    m, ctx = env
    keys = torch.zeros(4, dtype=torch.int64, device="cuda")
    slots = torch.arange(4, dtype=torch.int32, device="cuda")
    with pytest.raises(m.MqgError):
        m.mqg_select_row_candidates(ctx, keys, slots, 0)
    with pytest.raises(m.MqgError):
        m.mqg_select_row_candidates(ctx, keys, slots, 5)
    big = torch.zeros(257, dtype=torch.int64, device="cuda")
    with pytest.raises(m.MqgError):
        m.mqg_select_row_candidates(ctx, big, torch.zeros(257, dtype=torch.int32, device="cuda"), 3)
