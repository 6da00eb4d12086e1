"""Host-side logic that needs no GPU: the seeded input generators, the benchmark's command line,
the bindings' buffer bounds."""
import os
import subprocess
import sys

import numpy as np
import torch

from paper_2601_04707_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_chung_lu_graph_is_simple_symmetric_sorted_and_seeded():
    rp, ci = synth.chung_lu_graph(3000, 60_000, max_degree=500, seed=4)
    rp2, ci2 = synth.chung_lu_graph(3000, 60_000, max_degree=500, seed=4)
    assert torch.equal(rp, rp2) and torch.equal(ci, ci2)              # a pure function of its arguments
    rp3, ci3 = synth.chung_lu_graph(3000, 60_000, max_degree=500, seed=5)
    assert not (rp3.numel() == rp.numel() and ci3.numel() == ci.numel() and torch.equal(ci, ci3))
    rp, ci = rp.numpy(), ci.numpy()
    n = len(rp) - 1
    assert n == 3000 and rp[0] == 0 and rp[-1] == len(ci) and 0.85 * 60_000 < len(ci) <= 60_000
    src = np.repeat(np.arange(n), np.diff(rp))
    assert not np.any(src == ci)                                      # no self loops
    edges = set(zip(src.tolist(), ci.tolist()))
    assert len(edges) == len(ci)                                      # no multi-edges
    assert all((b, a) in edges for a, b in list(edges)[:5000])        # symmetric
    for v in range(0, n, 37):
        row = ci[rp[v]:rp[v + 1]]
        assert np.all(np.diff(row) > 0)                               # rows ascending
    deg = np.diff(rp)
    assert deg.max() <= 1.5 * 500 and deg.max() > 20 * np.median(deg)  # skewed, capped near the stated maximum
    # node ids are permuted: the degree is not monotone in the id
    assert abs(np.corrcoef(np.arange(n), deg)[0, 1]) < 0.1


def test_seed_batches_are_disjoint_slices_of_the_training_set():
    b = synth.seed_batches(1000, 64, 5, seed=2)
    assert len(b) == 5 and all(x.numel() == 64 and x.dtype == torch.int64 for x in b)
    allv = torch.cat(b)
    assert allv.unique().numel() == allv.numel() and int(allv.min()) >= 0 and int(allv.max()) < 1000
    assert all(torch.equal(x, y) for x, y in zip(b, synth.seed_batches(1000, 64, 5, seed=2)))
    part = synth.seed_batches(100_000, 64, 3, seed=2, train_fraction=0.01)
    train = torch.cat(part).unique()
    assert train.numel() == 3 * 64
    more = torch.cat(synth.seed_batches(100_000, 64, 15, seed=2, train_fraction=0.01))
    assert more.unique().numel() <= 1000                              # drawn from a 1 % training set, reused across epochs


def test_node_features_are_seeded_and_normal():
    a = synth.node_features(2000, 16, seed=1)
    assert torch.equal(a, synth.node_features(2000, 16, seed=1)) and a.dtype == torch.float32
    assert abs(float(a.mean())) < 0.05 and abs(float(a.std()) - 1.0) < 0.05
    h = synth.node_features(50, 8, dtype=torch.float16, seed=1)
    assert h.dtype == torch.float16 and h.shape == (50, 8)


def test_workloads_have_the_stated_shapes():
    w = synth.WORKLOADS
    assert (w["medium"].num_nodes, w["medium"].dim, w["medium"].fanouts, w["medium"].batch, w["medium"].cache_pct) == \
        (232_965, 602, [25, 10], 1024, 30)
    assert (w["large"].num_nodes, w["large"].fanouts, w["large"].cache_pct) == (2_449_029, [15, 10, 5], 20)
    assert w["xlarge"].num_nodes == 111_000_000 and w["xlarge"].feat_dtype == torch.float16 and w["xlarge"].train_fraction == 0.01
    assert w["stress"].batch == 8192 and w["stress"].in_flight == 4 and w["stress"].cache_sweep == [5, 20, 50]
    assert w["tiny"].cache_pct is None and w["tiny"].idx_dtype == torch.int32
    s = synth.scaled(w["large"], 0.01)
    assert s.fanouts == w["large"].fanouts and s.dim == w["large"].dim and s.batch == w["large"].batch
    assert abs(s.target_edges / s.num_nodes - w["large"].target_edges / w["large"].num_nodes) < 1.0


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "one GPU" in p.stderr and p.stdout.strip() == ""


def test_aligned_row_stride_rule():
    assert synth.aligned_row_stride(602, torch.float32) == 608          # 2,408 -> 2,432 bytes: +1 %
    assert synth.aligned_row_stride(100, torch.float32) == 100          # 400 bytes: 448 would be +12 %, stays 16-byte aligned
    assert synth.aligned_row_stride(128, torch.float16) == 128 and synth.aligned_row_stride(256, torch.float16) == 256
    assert synth.aligned_row_stride(7, torch.float32) == 8              # 28 -> 32 bytes (16-byte rule)
    for dim, dt in ((602, torch.float32), (100, torch.float32), (9, torch.float16), (1030, torch.float32)):
        st = synth.aligned_row_stride(dim, dt)
        elt = 2 if dt == torch.float16 else 4
        assert st >= dim and (st * elt) % 16 == 0
