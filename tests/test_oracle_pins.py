"""Pins for the CPU oracle: it is checked here against things other than itself -
published known-answer vectors, brute force written independently in Python,
closed forms, textbook special cases and library routines - so that a slip in
any of its functions (a dropped term, a wrong index, a wrong sign, a wrong
order) fails at least one test.  CPU only.
"""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from paper_2601_04707_amd import synth

M64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15
HERE = os.path.dirname(os.path.abspath(__file__))


# ------------------------------------------------------------ independent Python restatement

def py_mix(z):
    z &= M64
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & M64
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & M64
    z ^= z >> 31
    return z


def py_key(seed, layer, node, slot):
    h = py_mix((seed + GOLDEN) & M64)
    h = py_mix(h ^ layer)
    h = py_mix(h ^ node)
    return py_mix(h ^ slot)


def py_sample_row(seed, layer, node, d, k):
    if d <= k:
        return list(range(d))
    ranked = sorted((py_key(seed, layer, node, j), j) for j in range(d))
    return sorted(j for _, j in ranked[:k])


def py_sample_blocks(row_ptr, col_idx, seeds, fanouts, rng_seed):
    """Whole L-hop expansion with Python sets/dicts; returns list of dicts per block."""
    L = len(fanouts)
    blocks = [None] * L
    dst = [int(s) for s in seeds]
    for l in range(L - 1, -1, -1):
        rows = []
        for v in dst:
            s, e = int(row_ptr[v]), int(row_ptr[v + 1])
            slots = py_sample_row(rng_seed, l, v, e - s, fanouts[l])
            rows.append([int(col_idx[s + j]) for j in slots])
        dset = set(dst)
        new = sorted({u for r in rows for u in r} - dset)
        src = dst + new
        pos = {}
        for i, v in enumerate(src):
            pos.setdefault(v, i)
        indptr = [0]
        for r in rows:
            indptr.append(indptr[-1] + len(r))
        blocks[l] = dict(num_dst=len(dst), src=src, indptr=indptr,
                         indices=[pos[u] for r in rows for u in r],
                         nbr=[u for r in rows for u in r])
        dst = src
    return blocks


def tiny_graph(n=300, edges=3000, seed=0):
    rp, ci = synth.chung_lu_graph(n, edges, seed=seed)
    return rp.numpy(), ci.numpy()


# ------------------------------------------------------------ key function

def test_mix_matches_published_splitmix64_vectors():
    """golden/splitmix64_kat.txt: outputs of the public-domain SplitMix64 reference."""
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "splitmix64_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 8
    for seed, n, out in rows:
        state = (int(seed) + int(n) * GOLDEN) & M64
        assert oracle.mix(state) == int(out, 16)


def test_mix_is_a_bijection_on_small_domain_and_fixes_zero():
    assert oracle.mix(0) == 0
    outs = {oracle.mix(z) for z in range(1, 5000)}
    assert len(outs) == 4999 and 0 not in outs


def test_key_composition_matches_bigint_arithmetic():
    rng = np.random.default_rng(0)
    for _ in range(300):
        seed = int(rng.integers(0, 1 << 63)) * 2 + int(rng.integers(0, 2))
        layer = int(rng.integers(0, 8))
        node = int(rng.integers(0, 1 << 40))
        slot = int(rng.integers(0, 1 << 31))
        assert oracle.key(seed, layer, node, slot) == py_key(seed, layer, node, slot)
    # each coordinate matters
    base = oracle.key(5, 1, 7, 3)
    assert len({base, oracle.key(6, 1, 7, 3), oracle.key(5, 2, 7, 3), oracle.key(5, 1, 8, 3),
                oracle.key(5, 1, 7, 4)}) == 5


def test_keys_look_uniform():
    """Top byte of 64k consecutive-slot keys: chi-square against the flat law (255 dof)."""
    keys = np.array([oracle.key(42, 0, 17, j) for j in range(65536)], dtype=np.uint64)
    counts = np.bincount((keys >> np.uint64(56)).astype(np.int64), minlength=256)
    chi2 = ((counts - 256.0) ** 2 / 256.0).sum()
    assert chi2 < 255 + 6 * math.sqrt(2 * 255)
    low = np.bincount((keys & np.uint64(0xFF)).astype(np.int64), minlength=256)
    chi2 = ((low - 256.0) ** 2 / 256.0).sum()
    assert chi2 < 255 + 6 * math.sqrt(2 * 255)


# ------------------------------------------------------------ row selection

@pytest.mark.parametrize("d,k", [(1, 1), (3, 5), (5, 5), (6, 5), (7, 1), (40, 10), (64, 25),
                                 (65, 25), (300, 25), (2000, 15), (9, 64), (130, 64)])
def test_sample_row_equals_bruteforce_full_sort(d, k):
    for seed in (0, 1, 0xDEADBEEF, M64):
        for node in (0, 12345, 2**33 + 7):
            for layer in (0, 2):
                got = oracle.sample_row(seed, layer, node, d, k).tolist()
                want = py_sample_row(seed, layer, node, d, k)
                assert got == want
                assert len(got) == min(k, d) and len(set(got)) == len(got)
                assert got == sorted(got) and all(0 <= j < d for j in got)


def test_k_equals_one_is_argmin_of_keys():
    for node in range(50):
        d = 37
        keys = [py_key(9, 1, node, j) for j in range(d)]
        assert oracle.sample_row(9, 1, node, d, 1).tolist() == [int(np.argmin(np.array(keys, dtype=np.uint64)))]


@pytest.mark.parametrize("d,k", [(4, 2), (5, 2), (6, 3), (5, 4)])
def test_subsets_are_uniform(d, k):
    """Every k-subset of a short row appears with frequency 1/C(d,k) (4 sigma), and
    every slot is included with probability k/d."""
    trials = 60000
    subsets = {c: 0 for c in itertools.combinations(range(d), k)}
    incl = np.zeros(d)
    for s in range(trials):
        got = tuple(oracle.sample_row(s, 0, 11, d, k).tolist())
        subsets[got] += 1
        incl[list(got)] += 1
    p = 1.0 / len(subsets)
    sigma = math.sqrt(trials * p * (1 - p))
    for c, cnt in subsets.items():
        assert abs(cnt - trials * p) < 4.5 * sigma, (c, cnt, trials * p)
    q = k / d
    assert np.all(np.abs(incl - trials * q) < 4.5 * math.sqrt(trials * q * (1 - q)))


def test_resampled_per_layer_and_per_seed():
    a = oracle.sample_row(1, 0, 5, 200, 10).tolist()
    b = oracle.sample_row(1, 1, 5, 200, 10).tolist()
    c = oracle.sample_row(2, 0, 5, 200, 10).tolist()
    assert a != b and a != c


# ------------------------------------------------------------ blocks

@pytest.mark.parametrize("fanouts", [[3], [4, 2], [5, 3, 2], [64, 64]])
def test_blocks_equal_python_set_dict_bruteforce(fanouts):
    rp, ci = tiny_graph()
    seeds = synth.seed_batches(len(rp) - 1, 16, 1, seed=5)[0].numpy()
    for rng_seed in (0, 77):
        got = oracle.sample_blocks(rp, ci, seeds, fanouts, rng_seed)
        want = py_sample_blocks(rp, ci, seeds, fanouts, rng_seed)
        assert len(got) == len(fanouts)
        for g, w in zip(got, want):
            assert g.num_dst == w["num_dst"]
            assert g.src_ids.tolist() == w["src"]
            assert g.indptr.tolist() == w["indptr"]
            assert g.indices.tolist() == w["indices"]
            assert g.nbr_global.tolist() == w["nbr"]


def test_block_invariants():
    rp, ci = tiny_graph(2000, 40000, seed=3)
    n = len(rp) - 1
    seeds = synth.seed_batches(n, 64, 1, seed=9)[0].numpy()
    fanouts = [10, 5, 3]
    blocks = oracle.sample_blocks(rp, ci, seeds, fanouts, 123)
    dst = seeds
    for l in range(len(fanouts) - 1, -1, -1):
        b = blocks[l]
        nd = b.num_dst
        assert np.array_equal(b.src_ids[:nd], dst)                     # destinations are the prefix
        new = b.src_ids[nd:]
        assert np.all(np.diff(new) > 0)                                # strictly ascending
        assert len(np.intersect1d(new, dst)) == 0                      # disjoint from destinations
        assert len(np.unique(b.src_ids)) == b.num_src                  # relabel is a bijection
        assert np.array_equal(b.src_ids[b.indices], b.nbr_global)      # local -> global
        assert set(new.tolist()) == set(b.nbr_global.tolist()) - set(dst.tolist())
        for i, v in enumerate(dst):
            row = b.nbr_global[b.indptr[i]:b.indptr[i + 1]]
            adj = ci[rp[v]:rp[v + 1]]
            assert len(row) == min(fanouts[l], len(adj))               # min(fanout, degree)
            assert len(set(row.tolist())) == len(row)                  # distinct
            assert np.all(np.isin(row, adj))                           # true neighbours
            assert np.all(np.diff(np.searchsorted(adj, row)) > 0)      # ascending adjacency slot
        dst = b.src_ids


def test_full_fanout_is_exact_khop_expansion():
    """fanout >= max degree: blocks are the textbook frontier expansion (sparse A products)."""
    rp, ci = tiny_graph(400, 3000, seed=4)
    n = len(rp) - 1
    A = sp.csr_matrix((np.ones(len(ci)), ci, rp), shape=(n, n))
    maxdeg = int(np.diff(rp).max())
    seeds = np.array([3, 50, 7, 120], dtype=np.int64)
    blocks = oracle.sample_blocks(rp, ci, seeds, [maxdeg, maxdeg + 5], 1)
    reach = np.zeros(n)
    reach[seeds] = 1
    for l in (1, 0):
        b = blocks[l]
        reach = ((A.T @ reach) + reach > 0).astype(float)              # one more hop, keep self
        assert set(b.src_ids.tolist()) == set(np.nonzero(reach)[0].tolist())
        sub = A[b.src_ids[:b.num_dst]]
        assert np.array_equal(b.indptr, sub.indptr)
        assert np.array_equal(b.nbr_global, sub.indices)


def test_empty_rows_and_empty_batch():
    rp = np.array([0, 0, 2, 3, 3], dtype=np.int64)       # node 0 and 3 isolated
    ci = np.array([2, 3, 1], dtype=np.int64)             # (not symmetric on purpose: rows are in-neighbours)
    b = oracle.sample_blocks(rp, ci, np.array([0, 1], dtype=np.int64), [2, 2], 0)
    assert b[1].indptr.tolist() == [0, 0, 2] and b[1].src_ids.tolist() == [0, 1, 2, 3]
    assert b[0].num_dst == 4 and b[0].indptr.tolist() == [0, 0, 2, 3, 3]
    assert b[0].indices.tolist() == [2, 3, 1] and b[0].num_src == 4
    e = oracle.sample_blocks(rp, ci, np.array([], dtype=np.int64), [2], 0)
    assert e[0].num_dst == 0 and e[0].num_src == 0 and e[0].nnz == 0


# ------------------------------------------------------------ cache

def test_cache_equals_lexsort_bruteforce():
    rp, _ = tiny_graph(1000, 12000, seed=6)
    n = len(rp) - 1
    deg = np.diff(rp)
    order = np.lexsort((np.arange(n), -deg))             # degree descending, id ascending
    feats = np.random.default_rng(0).standard_normal((n, 7)).astype(np.float32)
    for num_cached in (0, 1, 137, n):
        c = oracle.build_cache(rp, num_cached, feats)
        assert np.array_equal(c.cached_ids, order[:num_cached])
        want = np.full(n, -1, dtype=np.int32)
        want[order[:num_cached]] = np.arange(num_cached, dtype=np.int32)
        assert np.array_equal(c.slot_of, want)
        assert np.array_equal(c.cache_rows, feats[order[:num_cached]])
    # ties: equal degrees go to the lower id
    rp2 = np.array([0, 2, 4, 6, 7], dtype=np.int64)
    assert oracle.build_cache(rp2, 2).cached_ids.tolist() == [0, 1]


def test_cache_covers_most_edge_endpoints_on_power_law_graph():
    """Skew argument of the paper's cache section: a small top-degree cache holds a much
    larger share of edge endpoints than of nodes."""
    rp, _ = tiny_graph(5000, 100000, seed=8)
    n = len(rp) - 1
    deg = np.diff(rp)
    c = oracle.build_cache(rp, n // 10)
    share = deg[c.cached_ids].sum() / deg.sum()
    assert share > 0.3


# ------------------------------------------------------------ gather

@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_gather_is_fancy_indexing_whatever_the_cache(dtype):
    rp, _ = tiny_graph(800, 9000, seed=2)
    n = len(rp) - 1
    rng = np.random.default_rng(1)
    feats = rng.standard_normal((n, 13)).astype(dtype)
    ids = rng.permutation(n)[:300].astype(np.int64)
    ref = feats[ids]
    out, h, m = oracle.gather(ids, feats, None)
    assert out.tobytes() == ref.tobytes() and (h, m) == (0, 300)
    for num_cached in (0, 80, n):
        c = oracle.build_cache(rp, num_cached, feats)
        out, h, m = oracle.gather(ids, feats, c)
        assert out.tobytes() == ref.tobytes()
        assert h == int((c.slot_of[ids] >= 0).sum()) and h + m == 300
    # a cache row that differs from the host row proves hits really read the cache
    c = oracle.build_cache(rp, 80, feats)
    c.cache_rows[:] = 0
    out, _, _ = oracle.gather(ids, feats, c)
    hit = c.slot_of[ids] >= 0
    assert np.all(out[hit] == 0) and out[~hit].tobytes() == ref[~hit].tobytes()


# ------------------------------------------------------------ fp16 helpers

def test_half_to_double_all_bit_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_float_to_half_rounds_to_nearest_even_like_numpy():
    rng = np.random.default_rng(3)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(5000) * 1e-6).astype(np.float32),      # subnormal halves
        (rng.standard_normal(5000) * 3e4).astype(np.float32),       # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 5.96e-8, 2.98e-8, 2.99e-8,
                  6.1e-5, 6.1035156e-5, 1.0009766, 1.0004883, 1.0014648, np.inf, -np.inf],
                 dtype=np.float32)])
    # exact ties between two halves
    h = rng.integers(0, 0x7BFF, 4000).astype(np.uint16)
    a = h.view(np.float16).astype(np.float64)
    b = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals = np.concatenate([vals, ((a + b) / 2).astype(np.float32)])
    with np.errstate(over="ignore"):
        want = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------------------ aggregate

def _random_block(rng, num_dst, num_src, max_row):
    counts = rng.integers(0, max_row + 1, num_dst)
    indptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    indices = rng.integers(0, num_src, indptr[-1]).astype(np.int32)
    return indptr, indices


@pytest.mark.parametrize("dtype,tol", [(np.float32, 1e-6), (np.float16, 1e-3)])
def test_mean_aggregate_equals_dense_row_normalised_product(dtype, tol):
    rng = np.random.default_rng(5)
    nd, ns, dim = 40, 90, 19
    indptr, indices = _random_block(rng, nd, ns, 7)
    x = rng.standard_normal((ns, dim)).astype(dtype)
    A = np.zeros((nd, ns))
    for i in range(nd):
        for e in range(indptr[i], indptr[i + 1]):
            A[i, indices[e]] += 1.0
    deg = A.sum(1, keepdims=True)
    want = np.where(deg > 0, (A @ x.astype(np.float64)) / np.maximum(deg, 1), 0.0)
    got = oracle.mean_aggregate(indptr, indices, x).astype(np.float64)
    assert np.allclose(got, want, rtol=tol, atol=tol)
    assert np.all(got[np.diff(indptr) == 0] == 0)                       # empty rows are zero
    # library routine: scipy CSR product
    S = sp.csr_matrix((np.ones(len(indices)), indices, indptr), shape=(nd, ns))
    want2 = (S @ x.astype(np.float64)) / np.maximum(np.diff(indptr), 1)[:, None]
    assert np.allclose(got, want2, rtol=tol, atol=tol)
    # fp32 result is the correctly rounded double mean
    if dtype == np.float32:
        assert np.array_equal(got.astype(np.float32), want.astype(np.float32))


def test_mean_aggregate_closed_forms():
    rng = np.random.default_rng(6)
    indptr, indices = _random_block(rng, 30, 50, 9)
    nonempty = np.diff(indptr) > 0
    const = np.full((50, 5), 3.25, dtype=np.float32)
    out = oracle.mean_aggregate(indptr, indices, const)
    assert np.all(out[nonempty] == 3.25) and np.all(out[~nonempty] == 0)
    # node-id features: the mean of the selected ids, exactly representable
    ids = np.arange(50, dtype=np.float32)[:, None] * np.array([[1.0, -2.0]], dtype=np.float32)
    out = oracle.mean_aggregate(indptr, indices, ids)
    for i in range(30):
        sel = indices[indptr[i]:indptr[i + 1]]
        if len(sel):
            assert out[i, 0] == np.float32(sel.astype(np.float64).mean())
            assert out[i, 1] == np.float32(-2.0 * sel.astype(np.float64).mean())
    # one-hot features reveal exactly which rows were summed and how often
    eye = np.eye(50, dtype=np.float32)
    out = oracle.mean_aggregate(indptr, indices, eye)
    for i in range(30):
        sel = indices[indptr[i]:indptr[i + 1]]
        if len(sel):
            want = np.bincount(sel, minlength=50) / len(sel)
            assert np.allclose(out[i], want, rtol=1e-7)


def test_full_fanout_aggregation_is_D_inv_A_X():
    rp, ci = tiny_graph(300, 2500, seed=7)
    n = len(rp) - 1
    x = np.random.default_rng(2).standard_normal((n, 6)).astype(np.float32)
    seeds = np.arange(0, n, 7, dtype=np.int64)
    b = oracle.sample_blocks(rp, ci, seeds, [int(np.diff(rp).max())], 0)[0]
    out = oracle.mean_aggregate(b.indptr, b.indices, x[b.src_ids])
    A = sp.csr_matrix((np.ones(len(ci)), ci, rp), shape=(n, n))
    deg = np.maximum(np.diff(rp), 1)[:, None]
    want = ((A @ x.astype(np.float64)) / deg)[seeds]
    assert np.allclose(out, want, rtol=1e-6, atol=1e-7)


def test_sampled_mean_is_unbiased_for_full_mean():
    """GraphSAGE paragraph of the paper: uniform neighbour sampling gives an unbiased
    estimate of the full-neighbourhood aggregate.  Average over many sampling seeds."""
    rp, ci = tiny_graph(200, 4000, seed=11)
    n = len(rp) - 1
    deg = np.diff(rp)
    v = int(np.argmax(deg))
    assert deg[v] > 20
    x = np.random.default_rng(4).standard_normal((n, 4))
    full = x[ci[rp[v]:rp[v + 1]]].mean(0)
    k, trials = 5, 4000
    acc = np.zeros(4)
    for s in range(trials):
        slots = oracle.sample_row(s, 0, v, int(deg[v]), k)
        acc += x[ci[rp[v] + slots]].mean(0)
    est = acc / trials
    # sd of one estimate <= sd(x)/sqrt(k); 5 sigma of the averaged estimate
    bound = 5 * x[ci[rp[v]:rp[v + 1]]].std(0) / math.sqrt(k * trials)
    assert np.all(np.abs(est - full) < bound)


# ------------------------------------------------------------ backward of the aggregation

@pytest.mark.parametrize("dtype,tol", [(np.float32, 1e-6), (np.float16, 2e-3)])
def test_backward_is_the_transposed_row_mean_operator(dtype, tol):
    rng = np.random.default_rng(8)
    nd, ns, dim = 60, 110, 9
    indptr, indices = _random_block(rng, nd, ns, 6)
    g = rng.standard_normal((nd, dim)).astype(dtype)
    M = np.zeros((nd, ns))
    for i in range(nd):
        for e in range(indptr[i], indptr[i + 1]):
            M[i, indices[e]] += 1.0 / (indptr[i + 1] - indptr[i])
    want = M.T @ g.astype(np.float64)
    got = oracle.mean_aggregate_backward(indptr, indices, ns, g).astype(np.float64)
    assert np.allclose(got, want, rtol=tol, atol=tol)
    # library routine: scipy's transposed CSR product
    S = sp.csr_matrix((np.repeat(1.0 / np.maximum(np.diff(indptr), 1), np.diff(indptr)), indices, indptr),
                      shape=(nd, ns))
    assert np.allclose(got, S.T @ g.astype(np.float64), rtol=tol, atol=tol)
    untouched = np.setdiff1d(np.arange(ns), indices)
    assert len(untouched) and np.all(got[untouched] == 0)
    if dtype == np.float32:
        assert np.array_equal(got.astype(np.float32), want.astype(np.float32))


def test_backward_is_adjoint_of_forward():
    """<M x, g> == <x, M^T g>: ties the backward oracle to the pinned forward oracle."""
    rng = np.random.default_rng(9)
    nd, ns, dim = 80, 150, 5
    indptr, indices = _random_block(rng, nd, ns, 8)
    x = rng.standard_normal((ns, dim)).astype(np.float32)
    g = rng.standard_normal((nd, dim)).astype(np.float32)
    fwd = oracle.mean_aggregate(indptr, indices, x).astype(np.float64)
    bwd = oracle.mean_aggregate_backward(indptr, indices, ns, g).astype(np.float64)
    lhs, rhs = (fwd * g).sum(), (x * bwd).sum()
    assert abs(lhs - rhs) < 1e-5 * max(1.0, abs(lhs))


def test_backward_closed_forms():
    indptr = np.array([0, 2, 2, 5], dtype=np.int64)             # row 1 is empty
    indices = np.array([0, 3, 3, 1, 0], dtype=np.int32)
    ones = np.ones((3, 2), dtype=np.float32)
    got = oracle.mean_aggregate_backward(indptr, indices, 5, ones)
    # source 0: 1/2 + 1/3, source 1: 1/3, source 3: 1/2 + 1/3, sources 2 and 4 untouched
    want = np.array([1 / 2 + 1 / 3, 1 / 3, 0, 1 / 2 + 1 / 3, 0])
    assert np.allclose(got[:, 0], want, rtol=1e-7) and np.array_equal(got[:, 0], got[:, 1])
    g = np.array([[6.0], [100.0], [9.0]], dtype=np.float32)      # the empty row's gradient goes nowhere
    got = oracle.mean_aggregate_backward(indptr, indices, 5, g)
    assert got[:, 0].tolist() == [6.0, 3.0, 0.0, 6.0, 0.0]


# ------------------------------------------------------------ sampled and random-walk cache

def test_sampled_cache_equals_python_restatement():
    rp, _ = tiny_graph(400, 5000, seed=12)
    n = len(rp) - 1
    for seed in (0, 99):
        keys = []
        for v in range(n):
            d = int(rp[v + 1] - rp[v])
            keys.append((min((py_key(seed, M64, v, j) for j in range(d)), default=M64), v))   # layer tag -1
        order = [v for _, v in sorted(keys)]
        for num_cached in (0, 1, 57, n):
            c = oracle.build_cache_sampled(rp, num_cached, seed)
            assert c.cached_ids.tolist() == order[:num_cached]
            want = np.full(n, -1, dtype=np.int32)
            want[order[:num_cached]] = np.arange(num_cached)
            assert np.array_equal(c.slot_of, want)
    assert oracle.build_cache_sampled(rp, 57, 1).cached_ids.tolist() != oracle.build_cache_sampled(rp, 57, 2).cached_ids.tolist()


def test_sampled_cache_is_weighted_sampling_without_replacement():
    """Eq. 13: membership probability proportional to in-degree.  On a 5-node degree sequence the
    first slot must be node a with probability w_a/W and every pair {a,b} must appear with the
    successive-sampling probability w_a/W*w_b/(W-w_a) + w_b/W*w_a/(W-w_b)."""
    w = np.array([1, 2, 3, 4, 2, 0])                              # node 5 has no neighbours
    rp = np.concatenate([[0], np.cumsum(w)]).astype(np.int64)
    W = w.sum()
    trials = 40000
    first = np.zeros(6)
    pairs = {}
    for seed in range(trials):
        ids = oracle.build_cache_sampled(rp, 2, seed).cached_ids.tolist()
        first[ids[0]] += 1
        key = tuple(sorted(ids))
        pairs[key] = pairs.get(key, 0) + 1
    p1 = w / W
    assert first[5] == 0
    assert np.all(np.abs(first - trials * p1) < 4.5 * np.sqrt(trials * p1 * (1 - p1)) + 1e-9)
    for a in range(5):
        for b in range(a + 1, 5):
            p = w[a] / W * w[b] / (W - w[a]) + w[b] / W * w[a] / (W - w[b])
            cnt = pairs.get((a, b), 0)
            assert abs(cnt - trials * p) < 4.5 * math.sqrt(trials * p * (1 - p)), (a, b, cnt, trials * p)


def directed_graph(n, edges, seed, keep=0.6):
    """A directed graph without self loops or repeated entries: a symmetric one with a random part
    of its edges dropped, so that most edges have no reverse."""
    rp, ci = tiny_graph(n, edges, seed=seed)
    rows = np.repeat(np.arange(n), np.diff(rp))
    mask = np.random.default_rng(seed).random(len(ci)) < keep
    rows, cols = rows[mask], ci[mask]
    rp2 = np.zeros(n + 1, dtype=np.int64)
    rp2[1:] = np.cumsum(np.bincount(rows, minlength=n))
    return rp2, cols.astype(np.int64)


def dense_walk(rp, ci, train, fanouts, how):
    """Eq. 14-15 with dense matrices: A[v, u] = 1 for u in row(v), D = diag(min(k, deg)/deg)."""
    n = len(rp) - 1
    A = np.zeros((n, n))
    for i in range(n):
        A[i, ci[rp[i]:rp[i + 1]]] = 1.0
    deg = np.diff(rp).astype(np.float64)
    P = np.zeros(n)
    P[train] = 1.0 / len(train)
    for k in fanouts:
        D = np.diag(np.where(deg > 0, np.minimum(k, deg) / np.maximum(deg, 1), 0.0))
        M = {"printed": D @ A + np.eye(n),            # Eq. 15 as printed, P a column vector
             "push": (D @ A + np.eye(n)).T,           # the same matrix along the sampling direction
             "pull": A @ D + np.eye(n)}[how]          # the neighbour's ratio, pulled along the rows
        P = M @ P
    return P


def test_random_walk_forms_equal_their_dense_matrix_statements():
    rp, ci = directed_graph(250, 2500, seed=13)
    train = np.array([3, 17, 100, 249, 42], dtype=np.int64)
    for fanouts in ([5], [5, 5], [4, 9, 2], [1000, 1000]):
        push = oracle.random_walk_scores(rp, ci, train, fanouts, oracle.WALK_PUSH)
        printed = oracle.random_walk_scores(rp, ci, train, fanouts, oracle.WALK_PRINTED)
        assert np.allclose(push, dense_walk(rp, ci, train, fanouts, "push"), rtol=1e-12, atol=1e-15)
        assert np.allclose(printed, dense_walk(rp, ci, train, fanouts, "printed"), rtol=1e-12, atol=1e-15)
        # on a directed graph the forms are three different things
        assert not np.allclose(push, printed, rtol=1e-3)
        assert not np.allclose(push, dense_walk(rp, ci, train, fanouts, "pull"), rtol=1e-3)
        if max(fanouts) < 1000:                                    # with D = I the printed form is the pull
            assert not np.allclose(printed, dense_walk(rp, ci, train, fanouts, "pull"), rtol=1e-3)
    assert np.array_equal(oracle.random_walk_scores(rp, ci, train, [5, 5]), oracle.random_walk_scores(rp, ci, train, [5, 5], 0))
    # fanout above every degree: D = I, the scores count walks, along the rows or against them
    n = len(rp) - 1
    A = np.zeros((n, n))
    for i in range(n):
        A[i, ci[rp[i]:rp[i + 1]]] = 1.0
    P0 = np.zeros(n)
    P0[train] = 1.0 / len(train)
    big = [10 ** 6, 10 ** 6]
    assert np.allclose(oracle.random_walk_scores(rp, ci, train, big, oracle.WALK_PRINTED),
                       np.linalg.matrix_power(A + np.eye(n), 2) @ P0, rtol=1e-12)
    assert np.allclose(oracle.random_walk_scores(rp, ci, train, big, oracle.WALK_PUSH),
                       np.linalg.matrix_power(A.T + np.eye(n), 2) @ P0, rtol=1e-12)
    # zero steps: the training distribution itself
    for form in (oracle.WALK_PUSH, oracle.WALK_PRINTED):
        assert np.array_equal(oracle.random_walk_scores(rp, ci, train, [], form), P0)
    with pytest.raises(ValueError):
        oracle.random_walk_scores(rp, ci, train, [5], 2)


def test_random_walk_push_on_a_symmetric_graph_is_the_neighbours_ratio_pulled():
    """On a graph that equals its transpose, "v hands d_v P[v] to the nodes it samples from" and
    "u collects d_v P[v] from its neighbours v" are one sum; with ascending rows even in the same
    order, so the two agree to the last bit."""
    rp, ci = tiny_graph(250, 2500, seed=13)
    n = len(rp) - 1
    deg = np.diff(rp).astype(np.float64)
    train = np.array([3, 17, 100, 249, 42], dtype=np.int64)
    fanouts = [4, 9, 2]
    got = oracle.random_walk_scores(rp, ci, train, fanouts, oracle.WALK_PUSH)
    assert np.allclose(got, dense_walk(rp, ci, train, fanouts, "pull"), rtol=1e-12, atol=1e-15)
    P = np.zeros(n)
    P[train] = 1.0 / len(train)
    for k in fanouts:                                              # the pull, row by row in adjacency order
        share = np.where(deg > 0, np.minimum(k, deg) / np.maximum(deg, 1), 0.0) * P
        nxt = P.copy()
        for u in range(n):
            acc = P[u]
            for v in ci[rp[u]:rp[u + 1]]:
                acc += share[v]
            nxt[u] = acc
        P = nxt
    assert np.array_equal(got, P)


def test_random_walk_worked_by_hand():
    # rows: 0:[1,2] 1:[0] 2:[0,3] 3:[]; training set {0}; fanout 1 -> d = [1/2, 1, 1/2, 0]
    rp = np.array([0, 2, 3, 5, 5], dtype=np.int64)
    ci = np.array([1, 2, 0, 0, 3], dtype=np.int64)
    # push: node 0 samples from {1, 2} and reaches each with 1/2; then 1 reaches 0 with 1/2 * 1, 2 reaches
    # 0 and 3 with 1/2 * 1/2 each - node 3 is sampled along 0 -> 2 -> 3
    assert oracle.random_walk_scores(rp, ci, [0], [1], oracle.WALK_PUSH).tolist() == [1.0, 0.5, 0.5, 0.0]
    assert oracle.random_walk_scores(rp, ci, [0], [1, 1], oracle.WALK_PUSH).tolist() == [1.75, 1.0, 1.0, 0.25]
    # as printed: node i collects d_i * (P over the nodes i samples from): 1 <- 1 * P[0], 2 <- 1/2 (P[0] + P[3])
    assert oracle.random_walk_scores(rp, ci, [0], [1], oracle.WALK_PRINTED).tolist() == [1.0, 1.0, 0.5, 0.0]
    assert oracle.random_walk_scores(rp, ci, [0], [1, 1], oracle.WALK_PRINTED).tolist() == [1.75, 2.0, 1.0, 0.0]
    # (the neighbour's ratio pulled along the rows would give [1.75, 1, 1, 0]: right on 0..2, blind to node 3)
    assert dense_walk(rp, ci, [0], [1, 1], "pull").tolist() == [1.75, 1.0, 1.0, 0.0]
    # a chain 0 -> 1 -> 2 (0 samples from 1, 1 from 2): only the push follows the sampling
    rp = np.array([0, 1, 2, 2], dtype=np.int64)
    ci = np.array([1, 2], dtype=np.int64)
    assert oracle.random_walk_scores(rp, ci, [0], [1, 1], oracle.WALK_PUSH).tolist() == [1.0, 2.0, 1.0]
    assert oracle.random_walk_scores(rp, ci, [0], [1, 1], oracle.WALK_PRINTED).tolist() == [1.0, 0.0, 0.0]
    # and from the far end the printed form walks back along the chain
    assert oracle.random_walk_scores(rp, ci, [2], [1, 1], oracle.WALK_PUSH).tolist() == [0.0, 0.0, 1.0]
    assert oracle.random_walk_scores(rp, ci, [2], [1, 1], oracle.WALK_PRINTED).tolist() == [1.0, 2.0, 1.0]


def test_random_walk_push_is_the_expected_frontier_of_node_wise_sampling():
    """Brute force over every outcome of the sampling process on a small directed graph, in exact
    rationals: start from a uniformly chosen training node; at step l every node of the frontier
    (a multiset) draws min(k_l, deg) distinct nodes of its row, every subset alike, and the drawn
    nodes join the frontier.  The push scores are the expected multiplicities; the printed form
    and the row-wise pull are not."""
    from fractions import Fraction
    rows = {0: [1, 2, 4], 1: [0, 3], 2: [3], 3: [4, 5, 0], 4: [], 5: [2, 1]}
    n = 6
    rp = np.zeros(n + 1, dtype=np.int64)
    rp[1:] = np.cumsum([len(rows[v]) for v in range(n)])
    ci = np.array([u for v in range(n) for u in rows[v]], dtype=np.int64)
    train, fanouts = [0, 5], [2, 1]

    def expand(frontier, k):
        """All (probability, next frontier) outcomes of one step."""
        per_node = []
        for v in frontier:
            subs = list(itertools.combinations(rows[v], min(k, len(rows[v]))))
            per_node.append([(Fraction(1, len(subs)), sub) for sub in subs])
        for combo in itertools.product(*per_node):
            pr = Fraction(1)
            nxt = list(frontier)
            for q, sub in combo:
                pr *= q
                nxt.extend(sub)
            yield pr, tuple(nxt)

    states = {(t,): Fraction(1, len(train)) for t in train}
    for k in fanouts:
        nxt_states = {}
        for fr, pr in states.items():
            for q, nf in expand(fr, k):
                nxt_states[nf] = nxt_states.get(nf, Fraction(0)) + pr * q
        states = nxt_states
    assert sum(states.values()) == 1
    expect = [sum(pr * fr.count(u) for fr, pr in states.items()) for u in range(n)]
    push = oracle.random_walk_scores(rp, ci, train, fanouts, oracle.WALK_PUSH)
    assert np.allclose(push, [float(x) for x in expect], rtol=1e-14, atol=0)
    assert not np.allclose(oracle.random_walk_scores(rp, ci, train, fanouts, oracle.WALK_PRINTED), push, rtol=1e-2)
    assert not np.allclose(dense_walk(rp, ci, train, fanouts, "pull"), push, rtol=1e-2)


def test_random_walk_push_follows_the_direction_of_the_sampler():
    """One step from a single node v, against the (pinned) block sampler on a directed graph: the
    mass that reaches u is the frequency with which sampling v draws u - u in row(v), never the
    nodes that merely list v."""
    rp, ci = directed_graph(60, 700, seed=3, keep=0.5)
    deg = np.diff(rp)
    v = int(np.argmax(deg))
    k = max(1, int(deg[v]) // 3)
    trials = 6000
    hits = np.zeros(60)
    for seed in range(trials):
        blk = oracle.sample_blocks(rp, ci, [v], [k], seed)[0]
        drawn = blk.src_ids[blk.indices]
        assert len(drawn) == k
        hits[drawn] += 1
    step = oracle.random_walk_scores(rp, ci, [v], [k], oracle.WALK_PUSH)
    step[v] -= 1.0                                                 # the "+ I" term
    p = step
    assert np.all(p[np.setdiff1d(np.arange(60), ci[rp[v]:rp[v + 1]])] == 0) and np.all(hits[p == 0] == 0)
    assert np.all(np.abs(hits - trials * p) <= 4.5 * np.sqrt(trials * p * (1 - p)) + 1e-9)
    listing_v = [u for u in range(60) if v in ci[rp[u]:rp[u + 1]] and u not in ci[rp[v]:rp[v + 1]]]
    assert listing_v                                               # the graph is directed here
    assert np.all(hits[listing_v] == 0)


def test_random_walk_scores_rank_reachable_hubs_first():
    """What the scores are for (cache section of the paper): nodes that sampling from the training
    set reaches with high probability.  With the whole graph as training set and one step the push
    score of node u is 1/N * (1 + sum over the nodes v that sample from u of min(k, deg_v)/deg_v),
    which grows with the number of such v - unlike the printed form, which gives every node of
    degree >= k the same 1 + k."""
    rp, ci = tiny_graph(600, 12000, seed=15)
    n = len(rp) - 1
    deg = np.diff(rp)
    sc = oracle.random_walk_scores(rp, ci, np.arange(n), [5], oracle.WALK_PUSH)
    big = deg >= 5
    assert np.unique(np.round(sc[big] * n, 9)).size > big.sum() // 2          # not one saturated value
    top = np.argsort(-sc)[:30]
    assert deg[top].mean() > 3 * deg.mean()
    printed = oracle.random_walk_scores(rp, ci, np.arange(n), [5], oracle.WALK_PRINTED)
    assert np.allclose(printed[big] * n, 6.0, rtol=1e-12)                      # saturated: 1 + k for all of them


def test_cache_by_score_equals_lexsort():
    rng = np.random.default_rng(14)
    scores = np.round(rng.random(500), 2)                        # many ties
    order = np.lexsort((np.arange(500), -scores))
    for num_cached in (0, 1, 123, 500):
        c = oracle.build_cache_by_score(scores, num_cached)
        assert np.array_equal(c.cached_ids, order[:num_cached])
        want = np.full(500, -1, dtype=np.int32)
        want[order[:num_cached]] = np.arange(num_cached)
        assert np.array_equal(c.slot_of, want)


# ------------------------------------------------------------------------- weighted (GCN) aggregation

def dense_gcn_operator(rp, ci):
    """P = D^-1/2 (A + I) D^-1/2 with D = row sums of A + I (Eq. 2), as a dense matrix."""
    n = len(rp) - 1
    A_hat = np.eye(n)
    for i in range(n):
        A_hat[i, ci[rp[i]:rp[i + 1]]] = 1.0
    d = A_hat.sum(axis=1)
    return A_hat / np.sqrt(np.outer(d, d))


def test_gcn_weights_with_whole_rows_reproduce_the_dense_operator():
    """Fanout above every degree: nothing is dropped, the factor of Eq. 3 is 1 and the block
    computes rows of P H exactly."""
    rp, ci = tiny_graph(60, 500, seed=21)
    n = len(rp) - 1
    P = dense_gcn_operator(rp, ci)
    assert np.allclose(P, P.T)
    rng = np.random.default_rng(2)
    H = rng.standard_normal((n, 7)).astype(np.float32)
    seeds = np.array([5, 0, 33, 59, 12], dtype=np.int64)
    blk = oracle.sample_blocks(rp, ci, seeds, [1000], 3)[0]
    ew, sw = oracle.gcn_edge_weights(rp, blk.src_ids, blk.indptr, blk.indices)
    for i, v in enumerate(seeds):
        assert sw[i] == pytest.approx(P[v, v], rel=1e-15)
        for p in range(blk.indptr[i], blk.indptr[i + 1]):
            assert ew[p] == pytest.approx(P[v, blk.src_ids[blk.indices[p]]], rel=1e-15)
    out = oracle.weighted_aggregate(blk.indptr, blk.indices, ew, sw, H[blk.src_ids])
    assert np.allclose(out, (P @ H.astype(np.float64))[seeds], rtol=2e-7, atol=1e-7)
    # without the diagonal term: (P - diag P) H
    out = oracle.weighted_aggregate(blk.indptr, blk.indices, ew, None, H[blk.src_ids])
    assert np.allclose(out, ((P - np.diag(np.diag(P))) @ H.astype(np.float64))[seeds], rtol=2e-7, atol=1e-7)


def test_gcn_estimator_is_unbiased_over_all_subsets():
    """Eq. 3: scaled by |N(v)| / s_node, the average over every possible sample of s_node
    neighbours equals the full row of P H (brute force over all subsets of one row)."""
    import itertools
    rp, ci = tiny_graph(40, 300, seed=22)
    deg = np.diff(rp)
    v = int(np.argmax((deg >= 6) & (deg <= 9)))
    assert 6 <= deg[v] <= 9
    P = dense_gcn_operator(rp, ci)
    rng = np.random.default_rng(4)
    H = rng.standard_normal((len(rp) - 1, 3)).astype(np.float32)
    nbrs = ci[rp[v]:rp[v + 1]]
    k = 3
    total = np.zeros(3)
    count = 0
    for sub in itertools.combinations(nbrs.tolist(), k):
        src_ids = np.array([v] + list(sub), dtype=np.int64)
        indptr = np.array([0, k], dtype=np.int64)
        indices = np.arange(1, k + 1, dtype=np.int32)
        ew, sw = oracle.gcn_edge_weights(rp, src_ids, indptr, indices)
        assert np.allclose(ew, deg[v] / k * P[v, list(sub)], rtol=1e-15)
        total += oracle.weighted_aggregate(indptr, indices, ew, sw, H[src_ids])[0].astype(np.float64)
        count += 1
    assert count == len(list(itertools.combinations(range(deg[v]), k)))
    assert np.allclose(total / count, (P @ H.astype(np.float64))[v], rtol=1e-6, atol=1e-6)


def test_weighted_aggregate_against_dense_product_and_its_transpose():
    rng = np.random.default_rng(23)
    nd, ns, dim = 30, 70, 5
    counts = rng.integers(0, 9, nd)
    indptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    indices = rng.integers(0, ns, indptr[-1]).astype(np.int32)          # repeated sources allowed
    ew = rng.standard_normal(indptr[-1])
    sw = rng.standard_normal(nd)
    M = np.zeros((nd, ns))
    for i in range(nd):
        M[i, i] += sw[i]
        for p in range(indptr[i], indptr[i + 1]):
            M[i, indices[p]] += ew[p]
    for dt, tol in ((np.float32, 1e-6), (np.float16, 2e-3)):
        x = rng.standard_normal((ns, dim)).astype(dt)
        g = rng.standard_normal((nd, dim)).astype(dt)
        out = oracle.weighted_aggregate(indptr, indices, ew, sw, x)
        assert out.dtype == dt and np.allclose(out, M @ x.astype(np.float64), rtol=tol, atol=tol)
        gx = oracle.weighted_aggregate_backward(indptr, indices, ns, ew, sw, g)
        assert gx.dtype == dt and np.allclose(gx, M.T @ g.astype(np.float64), rtol=tol, atol=tol)
    # equal weights 1/n_i and no diagonal: the mean aggregation
    x = rng.standard_normal((ns, dim)).astype(np.float32)
    n_i = np.repeat(np.maximum(counts, 1), counts)
    assert np.allclose(oracle.weighted_aggregate(indptr, indices, 1.0 / n_i, None, x),
                       oracle.mean_aggregate(indptr, indices, x), rtol=3e-7, atol=1e-7)


# ------------------------------------------------------------------------- draws with real weights

def test_exp_tickets_stream_is_the_scalar_functions_composed():
    got = oracle.exp_tickets(77, -3, 1000, 300)
    assert [int(x) for x in got] == [oracle.exp_ticket(oracle.key(77, -3, 1000 + i, 0)) for i in range(300)]


def test_exp_ticket_is_minus_log2_in_fixed_point():
    import math
    assert oracle.exp_ticket(1 << 63) == 1 << 32                 # r / 2^64 = 1/2
    for k in range(64):
        assert oracle.exp_ticket(1 << k) == (64 - k) << 32       # powers of two are exact
    assert oracle.exp_ticket(0) == oracle.exp_ticket(1) == 64 << 32
    assert 1 <= oracle.exp_ticket((1 << 64) - 1) <= 4            # -log2(1 - 2^-64) * 2^32, rounded up
    rng = np.random.default_rng(31)
    for r in rng.integers(1, 1 << 63, 3000, dtype=np.uint64).tolist() + [3, 5, 7, (1 << 64) - 12345, 3 << 62]:
        want = -math.log2(r / 2.0 ** 64) if r < (1 << 53) else 64 - math.log2(r)
        assert abs(oracle.exp_ticket(r) / 2.0 ** 32 - want) < 2.0 ** -28, r
    # monotone: a larger uniform never gives a larger ticket
    rs = np.sort(rng.integers(1, 1 << 63, 2000, dtype=np.uint64))
    t = [oracle.exp_ticket(int(r)) for r in rs]
    assert all(a >= b for a, b in zip(t, t[1:]))


def test_exp_tickets_are_exponentially_distributed():
    import math
    r = [oracle.key(7, 0, 0, j) for j in range(40000)]
    e = np.array([oracle.exp_ticket(x) for x in r]) * (math.log(2.0) / 2.0 ** 32)
    assert abs(e.mean() - 1.0) < 0.02 and abs(e.var() - 1.0) < 0.05
    for q in (0.1, 0.5, 0.9, 0.99):
        assert abs((e <= -math.log(1 - q)).mean() - q) < 0.01


def test_draw_by_score_matches_successive_sampling_probabilities():
    """Weighted sampling without replacement: the first pick is i with probability w_i / W, a pair
    {i, j} comes out with w_i/W * w_j/(W - w_i) + w_j/W * w_i/(W - w_j)."""
    w = np.array([1.0, 2.0, 3.0, 4.0, 10.0, 0.0])
    W = w.sum()
    trials = 30000
    first = np.zeros(6)
    pairs = {}
    for seed in range(trials):
        c = oracle.build_cache_drawn_by_score(w, 2, seed)
        first[c.cached_ids[0]] += 1
        key = tuple(sorted(c.cached_ids.tolist()))
        pairs[key] = pairs.get(key, 0) + 1
    assert first[5] == 0                                         # a zero score is never drawn
    p1 = w / W
    assert np.all(np.abs(first / trials - p1) < 4 * np.sqrt(p1 * (1 - p1) / trials) + 1e-9)
    for i in range(5):
        for j in range(i + 1, 5):
            p = w[i] / W * w[j] / (W - w[i]) + w[j] / W * w[i] / (W - w[j])
            assert abs(pairs.get((i, j), 0) / trials - p) < 4 * np.sqrt(p * (1 - p) / trials)


def test_draw_by_score_restated_with_numpy():
    rng = np.random.default_rng(33)
    sc = rng.random(400) ** 4
    sc[::9] = 0.0
    seed = 99
    t = np.array([oracle.exp_ticket(oracle.key(seed, -2, v, 0)) for v in range(400)], dtype=np.float64)
    with np.errstate(divide="ignore"):
        key = np.where(sc > 0, t / np.where(sc > 0, sc, 1.0), np.inf)
    order = np.lexsort((np.arange(400), key))
    for num_cached in (0, 1, 57, 400):
        c = oracle.build_cache_drawn_by_score(sc, num_cached, seed)
        assert np.array_equal(c.cached_ids, order[:num_cached])
        want = np.full(400, -1, dtype=np.int32)
        want[order[:num_cached]] = np.arange(num_cached)
        assert np.array_equal(c.slot_of, want)


# ------------------------------------------------------------------------- cache-prioritised sampling

def test_prioritised_row_equals_python_sort_and_keeps_cached_first():
    rng = np.random.default_rng(41)
    for trial in range(60):
        d = int(rng.integers(1, 200))
        k = int(rng.integers(1, 30))
        n = 500
        nbrs = rng.choice(n, size=d, replace=False)
        slot_of = np.where(rng.random(n) < rng.choice([0.0, 0.05, 0.3, 0.9, 1.0]), 7, -1).astype(np.int32)
        got = oracle.sample_row_prioritised(trial, 2, 11, nbrs, k, slot_of)
        if d <= k:
            assert got.tolist() == list(range(d))
            continue
        order = sorted(range(d), key=lambda j: (slot_of[nbrs[j]] < 0, oracle.key(trial, 2, 11, j), j))
        assert got.tolist() == sorted(order[:k])
        c = int((slot_of[nbrs] >= 0).sum())
        assert int((slot_of[nbrs[got]] >= 0).sum()) == min(k, c)
        # no cache at all, or everything cached: the plain uniform draw
        for so in (np.full(n, -1, np.int32), np.zeros(n, np.int32)):
            assert np.array_equal(oracle.sample_row_prioritised(trial, 2, 11, nbrs, k, so),
                                  oracle.sample_row(trial, 2, 11, d, k))


def test_prioritised_draw_is_uniform_within_each_class():
    d, k, n = 30, 6, 30
    nbrs = np.arange(n)
    slot_of = np.full(n, -1, np.int32)
    slot_of[:12] = 1                                             # 12 cached > k: only cached ones, k/12 each
    cnt = np.zeros(d)
    trials = 6000
    for s in range(trials):
        cnt[oracle.sample_row_prioritised(s, 0, 5, nbrs, k, slot_of)] += 1
    assert cnt[12:].sum() == 0
    p = k / 12
    assert np.all(np.abs(cnt[:12] / trials - p) < 4.5 * np.sqrt(p * (1 - p) / trials))
    slot_of[:] = -1
    slot_of[[3, 17]] = 1                                         # 2 cached < k: both always, the rest (k-2)/28 each
    cnt[:] = 0
    for s in range(trials):
        cnt[oracle.sample_row_prioritised(s, 0, 5, nbrs, k, slot_of)] += 1
    assert cnt[3] == trials and cnt[17] == trials
    rest = np.delete(cnt, [3, 17])
    p = (k - 2) / 28
    assert np.all(np.abs(rest / trials - p) < 4.5 * np.sqrt(p * (1 - p) / trials))


def test_prioritised_blocks_structure_and_fewer_uncached_sources():
    rp, ci = tiny_graph(3000, 90000, seed=42)
    n = len(rp) - 1
    cache = oracle.build_cache(rp, n // 5)
    seeds = np.random.default_rng(1).choice(n, 64, replace=False)
    plain = oracle.sample_blocks(rp, ci, seeds, [10, 5], 9)
    prio = oracle.sample_blocks(rp, ci, seeds, [10, 5], 9, prio_slot_of=cache.slot_of)
    for l in (1, 0):
        b = prio[l]
        dst = seeds if l == 1 else prio[1].src_ids
        assert np.array_equal(b.src_ids[:b.num_dst], dst)
        assert np.array_equal(np.diff(b.indptr), np.minimum(np.diff(rp)[dst], [10, 5][l]))
        assert np.array_equal(b.src_ids[b.indices], b.nbr_global)
        new = b.src_ids[b.num_dst:]
        assert np.all(np.diff(new) > 0) and not np.intersect1d(new, dst).size
        for i, v in enumerate(dst[:50]):                       # every sampled neighbour is a neighbour
            assert np.isin(b.nbr_global[b.indptr[i]:b.indptr[i + 1]], ci[rp[v]:rp[v + 1]]).all()
    unc = lambda blocks: int((cache.slot_of[blocks[0].src_ids] < 0).sum())
    assert unc(prio) < 0.7 * unc(plain)


# ------------------------------------------------------------------------- layer-wise sampling (LADIES)

def test_ladies_probabilities_equal_dense_column_norms():
    """Eq. 7 written with dense matrices: p_i = ||R P[:, i]||^2 / ||R P||_F^2."""
    rp, ci = tiny_graph(120, 1400, seed=51)
    P = dense_gcn_operator(rp, ci)
    rows = np.array([7, 0, 119, 33, 64, 90], dtype=np.int64)
    RP = P[rows]
    want = (RP ** 2).sum(axis=0) / (RP ** 2).sum()
    got = oracle.ladies_probabilities(rp, ci, rows)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-18) and abs(got.sum() - 1) < 1e-12
    # the integer masses of the block routine describe the same distribution
    b = oracle.ladies_blocks(rp, ci, rows, [10 ** 6], 1, want_mass=True)[0]
    deg1 = np.diff(rp) + 1
    m_py = np.zeros(120, dtype=object)
    for v in rows:
        add = (1 << 40) // int(deg1[v])
        m_py[v] += add
        for i in ci[rp[v]:rp[v + 1]]:
            m_py[i] += add
    assert [int(x) for x in b.mass] == [int(x) for x in m_py]
    q = b.mass.astype(np.float64) / deg1
    assert np.allclose(q / q.sum(), want, rtol=1e-9, atol=1e-18)
    # Eq. 6: the candidates are the rows' neighbours (and the rows themselves, from A + I)
    cand = set(rows.tolist())
    for v in rows:
        cand |= set(ci[rp[v]:rp[v + 1]].tolist())
    assert set(np.nonzero(b.mass)[0].tolist()) == cand and set(b.src_ids.tolist()) == cand


def test_ladies_block_with_every_candidate_reproduces_the_operator():
    """Layer size above the number of candidates: nothing is dropped; Eq. 8's scaling undone gives
    back P (weight * s * p_i == P_vi), and the normalised rows are P's rows divided by their sums."""
    rp, ci = tiny_graph(120, 1400, seed=52)
    P = dense_gcn_operator(rp, ci)
    rows = np.array([5, 17, 3, 80], dtype=np.int64)
    p = oracle.ladies_probabilities(rp, ci, rows)
    raw = oracle.ladies_blocks(rp, ci, rows, [10 ** 6], 4, normalise=False)[0]
    nrm = oracle.ladies_blocks(rp, ci, rows, [10 ** 6], 4, normalise=True)[0]
    s = raw.num_src
    assert np.all(np.diff(raw.src_ids) > 0)
    for t, v in enumerate(rows):
        e = slice(raw.indptr[t], raw.indptr[t + 1])
        ids = raw.src_ids[raw.indices[e]]
        assert ids[0] == v and ids[1:].tolist() == ci[rp[v]:rp[v + 1]].tolist()      # self edge, then slot order
        assert np.allclose(raw.edge_w[e] * s * p[ids], P[v, ids], rtol=1e-9)
        assert np.allclose(nrm.edge_w[e], P[v, ids] / p[ids] / (P[v, ids] / p[ids]).sum(), rtol=1e-9)
        assert abs(nrm.edge_w[e].sum() - 1.0) < 1e-12


def test_ladies_draw_restated_in_python_and_block_structure():
    rp, ci = tiny_graph(400, 6000, seed=53)
    n = len(rp) - 1
    deg1 = (np.diff(rp) + 1).astype(np.float64)
    seeds = np.random.default_rng(5).choice(n, 24, replace=False)
    sizes = [16, 40]
    blocks = oracle.ladies_blocks(rp, ci, seeds, sizes, 77, want_mass=True)
    dst = seeds
    for l in (1, 0):
        b = blocks[l]
        mass = b.mass
        cand = np.nonzero(mass)[0]
        assert len(cand) > sizes[l]
        t = np.array([oracle.exp_ticket(oracle.key(77, 64 + l, int(i), 0)) for i in cand], dtype=np.float64)
        key = (t * deg1[cand]) / mass[cand].astype(np.float64)
        order = np.lexsort((cand, key))
        assert np.array_equal(b.src_ids, np.sort(cand[order[:sizes[l]]]))
        assert b.num_dst == len(dst) and b.num_src == sizes[l]
        chosen = set(b.src_ids.tolist())
        for r, v in enumerate(dst):
            want = [v] * (int(v) in chosen) + [int(i) for i in ci[rp[v]:rp[v + 1]] if int(i) in chosen]
            got = b.src_ids[b.indices[b.indptr[r]:b.indptr[r + 1]]].tolist()
            assert got == want
            w = b.edge_w[b.indptr[r]:b.indptr[r + 1]]
            assert len(w) == 0 or abs(w.sum() - 1.0) < 1e-12
        dst = b.src_ids


def test_ladies_first_pick_follows_the_probabilities():
    rp, ci = tiny_graph(30, 120, seed=54)
    rows = np.array([2, 11, 20], dtype=np.int64)
    p = oracle.ladies_probabilities(rp, ci, rows)
    trials = 20000
    cnt = np.zeros(30)
    for seed in range(trials):
        cnt[oracle.ladies_blocks(rp, ci, rows, [1], seed)[0].src_ids[0]] += 1
    assert np.all(cnt[p == 0] == 0)
    assert np.all(np.abs(cnt / trials - p) < 4.5 * np.sqrt(p * (1 - p) / trials) + 1e-9)


def test_ladies_degenerate_cases():
    rp = np.array([0, 0, 2, 3, 3, 6], dtype=np.int64)            # nodes 0 and 3 have no neighbours
    ci = np.array([2, 4, 1, 0, 1, 2], dtype=np.int64)
    b = oracle.ladies_blocks(rp, ci, np.array([0], dtype=np.int64), [4], 1)[0]
    assert b.src_ids.tolist() == [0] and b.indices.tolist() == [0] and b.edge_w.tolist() == [1.0]
    b = oracle.ladies_blocks(rp, ci, np.zeros(0, dtype=np.int64), [4], 1)[0]
    assert b.num_src == 0 and b.nnz == 0 and b.indptr.tolist() == [0]
    b = oracle.ladies_blocks(rp, ci, np.array([1, 3], dtype=np.int64), [1], 3, normalise=False)[0]
    assert b.num_src == 1 and b.indptr[-1] == b.nnz


def test_fastgcn_probabilities_and_batch_independent_draw():
    rp, ci = tiny_graph(150, 1800, seed=55)
    n = len(rp) - 1
    P = dense_gcn_operator(rp, ci)
    want = (P ** 2).sum(axis=0) / (P ** 2).sum()                 # squared column norms of P itself
    assert np.allclose(oracle.ladies_probabilities(rp, ci), want, rtol=1e-12)
    a = oracle.ladies_blocks(rp, ci, np.array([3, 9, 27]), [20, 30], 5, fastgcn=True, want_mass=True)
    b = oracle.ladies_blocks(rp, ci, np.array([100, 4, 77, 12]), [20, 30], 5, fastgcn=True)
    deg1 = np.diff(rp) + 1
    q = a[1].mass.astype(np.float64) / deg1
    assert np.allclose(q / q.sum(), want, rtol=1e-9)
    for l in (0, 1):                                             # the draw does not look at the mini-batch
        assert np.array_equal(a[l].src_ids, b[l].src_ids) and a[l].num_src == [20, 30][l]
    # restated: race over all nodes
    t = np.array([oracle.exp_ticket(oracle.key(5, 64 + 1, i, 0)) for i in range(n)], dtype=np.float64)
    key = (t * deg1) / a[1].mass.astype(np.float64)
    assert np.array_equal(a[1].src_ids, np.sort(np.lexsort((np.arange(n), key))[:30]))
    # raw weights undo to P: weight * s * p_u == P_vu on the edges that survive
    raw = oracle.ladies_blocks(rp, ci, np.array([3, 9, 27]), [20, 30], 5, fastgcn=True, normalise=False)[1]
    for r, v in enumerate([3, 9, 27]):
        e = slice(raw.indptr[r], raw.indptr[r + 1])
        ids = raw.src_ids[raw.indices[e]]
        assert np.allclose(raw.edge_w[e] * 30 * want[ids], P[v, ids], rtol=1e-9)
        assert set(ids.tolist()) == (set(ci[rp[v]:rp[v + 1]].tolist()) | {v}) & set(raw.src_ids.tolist())


# ------------------------------------------------------------------------- "flat" probabilities (Eq. 10)

def test_flat_probabilities_are_the_column_norms_and_minimise_the_variance():
    """p_i proportional to ||R P[:, i]|| (not squared).  Pinned by the dense norms and by what the
    paper gives as their reason: with rows of H W of equal norm, this p minimises the variance
    sum_i ||R P[:, i]||^2 ||(HW)_i||^2 / p_i of the sampled product over all distributions - checked
    against the squared-norm probabilities, the uniform ones and random perturbations."""
    rp, ci = tiny_graph(120, 1400, seed=61)
    P = dense_gcn_operator(rp, ci)
    rows = np.array([7, 0, 119, 33, 64, 90], dtype=np.int64)
    norms = np.sqrt((P[rows] ** 2).sum(axis=0))
    want = norms / norms.sum()
    got = oracle.ladies_probabilities(rp, ci, rows, flat=True)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-18) and abs(got.sum() - 1) < 1e-12
    assert np.allclose(oracle.ladies_probabilities(rp, ci, flat=True),
                       np.sqrt((P ** 2).sum(axis=0)) / np.sqrt((P ** 2).sum(axis=0)).sum(), rtol=1e-12)
    support = norms > 0
    variance = lambda p: float((norms[support] ** 2 / p[support]).sum())
    best = variance(got)
    squared = oracle.ladies_probabilities(rp, ci, rows)
    uniform = support / support.sum()
    assert best < variance(squared) and best < variance(uniform)
    rng = np.random.default_rng(0)
    for _ in range(200):
        q = got * np.exp(0.2 * rng.standard_normal(len(got)))
        assert best <= variance(q / q[support].sum()) + 1e-12


def test_flat_draw_restated_first_pick_and_weights():
    rp, ci = tiny_graph(400, 6000, seed=62)
    n = len(rp) - 1
    deg1 = (np.diff(rp) + 1).astype(np.float64)
    seeds = np.random.default_rng(5).choice(n, 24, replace=False)
    # the draw: squared tickets over q, i.e. tickets over sqrt(q)
    b = oracle.ladies_blocks(rp, ci, seeds, [40], 77, want_mass=True, flat=True, normalise=False)[0]
    cand = np.nonzero(b.mass)[0]
    t = np.array([oracle.exp_ticket(oracle.key(77, 64, int(i), 0)) for i in cand], dtype=np.float64)
    key = ((t * t) * deg1[cand]) / b.mass[cand].astype(np.float64)
    assert np.array_equal(b.src_ids, np.sort(cand[np.lexsort((cand, key))[:40]]))
    exact = [(int(oracle.exp_ticket(oracle.key(77, 64, int(i), 0))) ** 2 * (int(deg1[i])), int(b.mass[i])) for i in cand]
    from fractions import Fraction
    order_exact = sorted(range(len(cand)), key=lambda c: (Fraction(exact[c][0], exact[c][1]), int(cand[c])))
    assert np.array_equal(b.src_ids, np.sort(cand[order_exact[:40]]))        # double rounding changes no decision here
    plain = oracle.ladies_blocks(rp, ci, seeds, [40], 77)[0]
    assert not np.array_equal(plain.src_ids, b.src_ids)                      # another distribution than Eq. 7's
    # weights: P_vi / (s p_i) with the flat p
    P = dense_gcn_operator(rp, ci)
    p = oracle.ladies_probabilities(rp, ci, seeds, flat=True)
    for r, v in enumerate(seeds):
        e = slice(b.indptr[r], b.indptr[r + 1])
        ids = b.src_ids[b.indices[e]]
        assert np.allclose(b.edge_w[e] * 40 * p[ids], P[v, ids], rtol=1e-9)


def test_flat_first_pick_follows_the_flat_probabilities():
    rp, ci = tiny_graph(30, 120, seed=54)
    rows = np.array([2, 11, 20], dtype=np.int64)
    p = oracle.ladies_probabilities(rp, ci, rows, flat=True)
    p2 = oracle.ladies_probabilities(rp, ci, rows)
    assert np.abs(p - p2).max() > 0.02                                      # the two distributions differ visibly
    trials = 20000
    cnt = np.zeros(30)
    for seed in range(trials):
        cnt[oracle.ladies_blocks(rp, ci, rows, [1], seed, flat=True)[0].src_ids[0]] += 1
    assert np.all(cnt[p == 0] == 0)
    assert np.all(np.abs(cnt / trials - p) < 4.5 * np.sqrt(p * (1 - p) / trials) + 1e-9)
    assert np.any(np.abs(cnt / trials - p2) > 6 * np.sqrt(p2 * (1 - p2) / trials))   # and not Eq. 7's


def test_flat_with_equal_norms_draws_as_the_plain_method_and_combines_with_debias():
    # a cycle: every column of P has the same norm, so squaring the tickets changes no order
    n = 40
    rp = np.arange(0, 2 * n + 1, 2, dtype=np.int64)
    ci = np.array([[(v - 1) % n, (v + 1) % n] for v in range(n)], dtype=np.int64).reshape(-1)
    seeds = np.arange(0, n, 3, dtype=np.int64)
    a = oracle.ladies_blocks(rp, ci, seeds, [12], 3, fastgcn=True)[0]
    b = oracle.ladies_blocks(rp, ci, seeds, [12], 3, fastgcn=True, flat=True)[0]
    assert np.array_equal(a.src_ids, b.src_ids) and np.allclose(a.edge_w, b.edge_w, rtol=1e-12)
    # flat + debias: the coefficients are those of Eq. 12 for the flat probabilities in race order
    rp2, ci2 = tiny_graph(200, 2400, seed=63)
    rows = np.random.default_rng(2).choice(200, 16, replace=False)
    blk = oracle.ladies_blocks(rp2, ci2, rows, [25], 9, flat=True, debias=True, normalise=False, want_mass=True)[0]
    deg1 = (np.diff(rp2) + 1).astype(np.float64)
    cand = np.nonzero(blk.mass)[0]
    t = np.array([oracle.exp_ticket(oracle.key(9, 64, int(i), 0)) for i in cand], dtype=np.float64)
    key = ((t * t) * deg1[cand]) / blk.mass[cand].astype(np.float64)
    drawn = cand[np.lexsort((cand, key))[:25]]
    p = oracle.ladies_probabilities(rp2, ci2, rows, flat=True)
    beta = oracle.debias_coefficients(p[drawn], len(cand))
    beta_of = dict(zip(drawn.tolist(), beta.tolist()))
    P = dense_gcn_operator(rp2, ci2)
    for r, v in enumerate(rows):
        e = slice(blk.indptr[r], blk.indptr[r + 1])
        ids = blk.src_ids[blk.indices[e]]
        assert np.allclose(blk.edge_w[e], [P[v, i] * beta_of[int(i)] for i in ids], rtol=1e-9)


# ------------------------------------------------------------------------- debiased coefficients (Eq. 12)

def test_debias_coefficients_closed_forms():
    n = 9
    for s in range(1, n + 1):                                    # equal probabilities: simple random sampling, n / s each
        beta = oracle.debias_coefficients(np.full(s, 1.0 / n), n)
        assert np.allclose(beta, n / s, rtol=1e-12), s
    rng = np.random.default_rng(61)
    p = rng.random(7)
    p /= p.sum()
    beta = oracle.debias_coefficients(p[rng.permutation(7)], 7)   # everything drawn: the plain sum
    assert np.allclose(beta, 1.0, rtol=1e-9)
    assert oracle.debias_coefficients(p[:1], 7)[0] == pytest.approx(1.0 / p[0])   # one draw: X / p


def test_debias_estimator_is_unbiased_over_all_ordered_draws():
    """Brute force: every ordered sample of s of n items with its successive-sampling probability;
    the expectation of sum_j beta_j X_j is the population total, for unequal probabilities."""
    import itertools
    p = np.array([0.05, 0.1, 0.15, 0.3, 0.4])
    X = np.array([3.0, -1.0, 7.0, 2.5, -4.0])
    n = 5
    for s in (1, 2, 3, 4):
        expect = 0.0
        total_prob = 0.0
        for order in itertools.permutations(range(n), s):
            prob, rest = 1.0, 1.0
            for i in order:
                prob *= p[i] / rest
                rest -= p[i]
            beta = oracle.debias_coefficients(p[list(order)], n)
            expect += prob * float(beta @ X[list(order)])
            total_prob += prob
        assert abs(total_prob - 1.0) < 1e-12
        assert abs(expect - X.sum()) < 1e-10, s
    # the plain importance weights 1 / (s p) are biased under the same draws (what Eq. 12 repairs)
    s = 3
    expect = 0.0
    for order in itertools.permutations(range(n), s):
        prob, rest = 1.0, 1.0
        for i in order:
            prob *= p[i] / rest
            rest -= p[i]
        expect += prob * float((X[list(order)] / (s * p[list(order)])).sum())
    assert abs(expect - X.sum()) > 0.1


def test_debiased_layerwise_blocks():
    rp, ci = tiny_graph(400, 6000, seed=62)
    n = len(rp) - 1
    P = dense_gcn_operator(rp, ci)
    seeds = np.random.default_rng(6).choice(n, 20, replace=False)
    for fastgcn in (False, True):
        plain = oracle.ladies_blocks(rp, ci, seeds, [30], 3, normalise=False, fastgcn=fastgcn, want_mass=True)[0]
        deb = oracle.ladies_blocks(rp, ci, seeds, [30], 3, normalise=False, fastgcn=fastgcn, debias=True)[0]
        assert np.array_equal(plain.src_ids, deb.src_ids) and np.array_equal(plain.indices, deb.indices)
        # restated: race order, probabilities, coefficients
        deg1 = (np.diff(rp) + 1).astype(np.float64)
        cand = np.nonzero(plain.mass)[0]
        t = np.array([oracle.exp_ticket(oracle.key(3, 64, int(i), 0)) for i in cand], dtype=np.float64)
        key = (t * deg1[cand]) / plain.mass[cand].astype(np.float64)
        order = cand[np.lexsort((cand, key))[:30]]
        q = plain.mass[cand].astype(np.float64) / deg1[cand]
        p_of = dict(zip(cand.tolist(), (q / q.sum()).tolist()))
        beta = oracle.debias_coefficients([p_of[int(i)] for i in order], len(cand))
        beta_of = dict(zip(order.tolist(), beta.tolist()))
        for r, v in enumerate(seeds):
            e = slice(deb.indptr[r], deb.indptr[r + 1])
            ids = deb.src_ids[deb.indices[e]]
            assert np.allclose(deb.edge_w[e], [P[v, i] * beta_of[int(i)] for i in ids], rtol=1e-9)
    # every candidate drawn: coefficients 1, the block is P restricted to the rows
    allc = oracle.ladies_blocks(rp, ci, seeds, [10 ** 6], 3, normalise=False, debias=True)[0]
    for r, v in enumerate(seeds):
        e = slice(allc.indptr[r], allc.indptr[r + 1])
        assert np.allclose(allc.edge_w[e], P[v, allc.src_ids[allc.indices[e]]], rtol=1e-12)
