"""Helpers of the GPU parity tests: run the HIP path through the C ABI and bring the
results back as numpy arrays in the oracle's layout."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2601_04707_amd import synth


def to_dev(t):
    return t.to("cuda").contiguous()


def hip_sample(mqg, ctx, graph, blocks, seeds_cpu, fanouts, rng_seed):
    """Returns a list (by block) of dicts with numpy num_dst/src_ids/indptr/indices."""
    seeds = to_dev(seeds_cpu.to(graph.idx_dtype))
    mqg.mqg_sample_blocks(ctx, graph, seeds, fanouts, rng_seed, blocks)
    torch.cuda.synchronize()
    sizes = blocks.host_sizes()
    out = []
    for l in range(len(fanouts)):
        nd, ns, nnz, flags = sizes[l]
        assert flags == 0
        out.append(dict(num_dst=nd, num_src=ns, nnz=nnz,
                        src_ids=blocks.src_ids[l][:ns].cpu().numpy().astype(np.int64),
                        indptr=blocks.indptr[l][:nd + 1].cpu().numpy().astype(np.int64),
                        indices=blocks.indices[l][:nnz].cpu().numpy()))
    return out


def assert_blocks_equal(got, want):
    """got: hip_sample output; want: list of oracle.Block.  Bit-exact."""
    assert len(got) == len(want)
    for l, (g, w) in enumerate(zip(got, want)):
        assert g["num_dst"] == w.num_dst, f"block {l}: num_dst {g['num_dst']} != {w.num_dst}"
        assert g["num_src"] == w.num_src, f"block {l}: num_src {g['num_src']} != {w.num_src}"
        assert g["nnz"] == w.nnz, f"block {l}: nnz {g['nnz']} != {w.nnz}"
        assert np.array_equal(g["indptr"], w.indptr), f"block {l}: indptr differs"
        assert np.array_equal(g["src_ids"], w.src_ids), f"block {l}: src_ids differ"
        assert np.array_equal(g["indices"], w.indices), f"block {l}: indices differ"


def agg_tolerance_ok(got, ref, x_abs_mean, tol):
    """|got - ref| <= tol * max(|ref|, mean |x|) element-wise: the forward error of a sum
    scales with the magnitude of its terms, and means of N(0,1) rows are often near zero."""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    bound = tol * np.maximum(np.abs(ref), x_abs_mean)
    return np.all(np.abs(got - ref) <= bound), float(np.max(np.abs(got - ref) / np.maximum(bound, 1e-300)))


def make_graph(workload, seed=0, device="cuda"):
    rp, ci = synth.build_graph(workload, seed=seed, device=device)
    return rp, ci
