"""Weights of the sampled graph-convolution estimator (paper Eq. 1-3) and weighted aggregation,
forward and backward, on the GPU versus the oracle, through the C ABI.

Tolerances.  Weights: the kernel computes in double and rounds once, so it must agree with the
oracle's double to one float rounding (6e-8 relative; 1.2e-7 allowed for the square root's last
bit).  Sums: |gpu - oracle| <= tol * max(|oracle|, mass), tol = 1e-5 (fp32) / 2e-3 (fp16), mass =
mean|x| * sum of |weights| of the row: fp32 accumulation error scales with the terms added.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_04707_amd import synth
from gpu_util import hip_sample, to_dev

pytestmark = pytest.mark.gpu

TOL = {np.float32: 1e-5, np.float16: 2e-3}


@pytest.fixture(scope="module")
def mqg():
    from paper_2601_04707_amd import mqg as m
    assert torch.cuda.is_available()
    return m


def bare_blocks(mqg, indptr, indices, nd, ns):
    rp = torch.tensor([0, 0], dtype=torch.int64)
    g = mqg.Graph(to_dev(rp), torch.zeros(1, dtype=torch.int64, device="cuda"))
    ctx = mqg.Context(g, 1, [1])
    blocks = mqg.Blocks(g, 1, [1])
    nnz = int(indptr[-1])
    ip = to_dev(torch.from_numpy(indptr.astype(np.int32)))
    ix = torch.zeros(max(nnz, 1), dtype=torch.int32, device="cuda")
    ix[:nnz] = torch.from_numpy(indices.astype(np.int32)).cuda()
    sizes = torch.tensor([nd, ns, nnz, 0], dtype=torch.int64, device="cuda")
    blocks.c[0] = mqg.CBlock(nd, ns, max(nnz, 1), None, ip.data_ptr(), ix.data_ptr(), sizes.data_ptr())
    blocks.bounds[0] = (nd, ns, max(nnz, 1))
    blocks._keep = (ip, ix, sizes, g)
    return ctx, blocks


def check(got, ref, mass, tol):
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = tol * np.maximum(np.abs(ref.astype(np.float64)), mass[:, None])
    assert np.all(err <= bound), float((err / np.maximum(bound, 1e-300)).max())


def row_mass(indptr, ew, sw, x):
    m = np.add.reduceat(np.concatenate([np.abs(ew), [0.0]]), np.minimum(indptr[:-1], len(ew))) * (np.diff(indptr) > 0)
    if sw is not None:
        m = m + np.abs(sw)
    return m * float(np.abs(x.astype(np.float64)).mean())


def random_block(rng, nd=900, ns=2500):
    counts = rng.integers(0, 26, nd)
    counts[::40] = 0
    indptr = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    p = 1.0 / (np.arange(ns) + 5.0) ** 1.2
    p[ns // 2:] = 0
    p /= p.sum()
    indices = np.concatenate([rng.choice(ns, size=c, replace=False, p=p) for c in counts]).astype(np.int32)
    return indptr, indices


@pytest.mark.parametrize("dim,dtype", [(64, np.float32), (100, np.float32), (602, np.float32), (128, np.float16),
                                       (256, np.float16), (7, np.float32), (9, np.float16), (1030, np.float32)])
@pytest.mark.parametrize("with_self", [True, False])
def test_weighted_forward_and_backward_random_blocks(mqg, dim, dtype, with_self):
    rng = np.random.default_rng(dim + 7)
    nd, ns = 900, 2500
    indptr, indices = random_block(rng, nd, ns)
    nnz = int(indptr[-1])
    ew = rng.standard_normal(nnz).astype(np.float32)            # signed weights
    sw = rng.standard_normal(nd).astype(np.float32) if with_self else None
    if with_self:
        sw[::7] = 0.0
    x = rng.standard_normal((ns, dim)).astype(dtype)
    g = rng.standard_normal((nd, dim)).astype(dtype)
    ctx, blocks = bare_blocks(mqg, indptr, indices, nd, ns)
    ew_d = to_dev(torch.from_numpy(ew))
    sw_d = to_dev(torch.from_numpy(sw)) if with_self else None
    # forward
    ref = oracle.weighted_aggregate(indptr, indices, ew, sw, x)
    xd = to_dev(torch.from_numpy(x))
    out = torch.full((nd + 2, dim), 5.0, dtype=xd.dtype, device="cuda")
    mqg.mqg_weighted_aggregate(ctx, blocks, 0, ew_d, sw_d, xd, out)
    torch.cuda.synchronize()
    check(out[:nd].cpu().numpy(), ref, row_mass(indptr, ew, sw, x), TOL[dtype])
    assert torch.all(out[nd:] == 5.0)
    # backward
    refb = oracle.weighted_aggregate_backward(indptr, indices, ns, ew, sw, g)
    gd = to_dev(torch.from_numpy(g))
    gx = torch.full((ns + 3, dim), 9.0, dtype=gd.dtype, device="cuda")
    mqg.mqg_weighted_aggregate_backward(ctx, blocks, 0, ew_d, sw_d, gd, gx)
    torch.cuda.synchronize()
    mass = np.bincount(indices, weights=np.abs(ew), minlength=ns)
    if with_self:
        mass[:nd] += np.abs(sw)
    check(gx[:ns].cpu().numpy(), refb, mass * float(np.abs(g.astype(np.float64)).mean()), TOL[dtype])
    assert torch.all(gx[ns:] == 9.0)
    gx2 = torch.zeros_like(gx)                                   # reproducible bit for bit
    mqg.mqg_weighted_aggregate_backward(ctx, blocks, 0, ew_d, sw_d, gd, gx2)
    torch.cuda.synchronize()
    assert torch.equal(gx2[:ns], gx[:ns])
    # the mean aggregation's backward still works on the same context afterwards (shared scratch)
    gm = torch.zeros_like(gx)
    mqg.mqg_sage_mean_aggregate_backward(ctx, blocks, 0, gd, gm)
    torch.cuda.synchronize()
    refm = oracle.mean_aggregate_backward(indptr, indices, ns, g)
    n_i = np.repeat(np.maximum(np.diff(indptr), 1), np.diff(indptr))
    massm = np.bincount(indices, weights=1.0 / n_i, minlength=ns) * float(np.abs(g.astype(np.float64)).mean())
    check(gm[:ns].cpu().numpy(), refm, massm, TOL[dtype])


def test_weighted_small_cases_by_hand(mqg):
    indptr = np.array([0, 2, 2, 5], dtype=np.int64)
    indices = np.array([0, 3, 3, 1, 0], dtype=np.int32)
    ctx, blocks = bare_blocks(mqg, indptr, indices, 3, 5)
    ew = torch.tensor([0.5, 2.0, 1.0, -1.0, 4.0], device="cuda")
    sw = torch.tensor([10.0, 100.0, 0.0], device="cuda")
    x = torch.tensor([[1.0], [2.0], [3.0], [4.0], [5.0]], device="cuda")
    out = torch.zeros((3, 1), device="cuda")
    mqg.mqg_weighted_aggregate(ctx, blocks, 0, ew, sw, x, out)
    torch.cuda.synchronize()
    assert out[:, 0].tolist() == [10.0 + 0.5 + 8.0, 200.0, 4.0 - 2.0 + 4.0]
    mqg.mqg_weighted_aggregate(ctx, blocks, 0, ew, None, x, out)
    torch.cuda.synchronize()
    assert out[:, 0].tolist() == [8.5, 0.0, 6.0]
    g = torch.tensor([[1.0], [10.0], [100.0]], device="cuda")
    gx = torch.full((5, 1), 7.0, device="cuda")
    mqg.mqg_weighted_aggregate_backward(ctx, blocks, 0, ew, sw, g, gx)
    torch.cuda.synchronize()
    assert gx[:, 0].tolist() == [10.0 + 0.5 + 400.0, 1000.0 - 100.0, 0.0, 2.0 + 100.0, 0.0]
    # an empty block
    ctx, blocks = bare_blocks(mqg, np.array([0, 0, 0], dtype=np.int64), np.zeros(0, np.int32), 2, 4)
    ew = torch.zeros(1, device="cuda")
    out = torch.full((2, 3), 3.0, device="cuda")
    mqg.mqg_weighted_aggregate(ctx, blocks, 0, ew, None, torch.ones((4, 3), device="cuda"), out)
    gx = torch.full((4, 3), 3.0, device="cuda")
    mqg.mqg_weighted_aggregate_backward(ctx, blocks, 0, ew, None, torch.ones((2, 3), device="cuda"), gx)
    torch.cuda.synchronize()
    assert torch.all(out == 0) and torch.all(gx == 0)


@pytest.mark.parametrize("ptr,idx", [(torch.int32, torch.int32), (torch.int64, torch.int64), (torch.int64, torch.int32)])
def test_gcn_weights_and_estimator_on_sampled_blocks(mqg, ptr, idx):
    rp, ci = synth.chung_lu_graph(20000, 400_000, max_degree=3000, seed=1)
    rp, ci = rp.to(ptr), ci.to(idx)
    g = mqg.Graph(to_dev(rp), to_dev(ci))
    fanouts = [15, 10, 5]
    batch, dim = 300, 48
    ctx = mqg.Context(g, batch, fanouts)
    blocks = mqg.Blocks(g, batch, fanouts)
    seeds = synth.seed_batches(rp.numel() - 1, batch, 1, seed=5)[0]
    got_blocks = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 77)
    rp_np = rp.numpy().astype(np.int64)
    rng = np.random.default_rng(3)
    for l in range(3):
        b = got_blocks[l]
        nd, ns, nnz = b["num_dst"], b["num_src"], b["nnz"]
        ew_ref, sw_ref = oracle.gcn_edge_weights(rp_np, b["src_ids"], b["indptr"], b["indices"])
        ew = torch.full((blocks.bounds[l][2] + 1,), -1.0, device="cuda")
        sw = torch.full((blocks.bounds[l][0] + 1,), -1.0, device="cuda")
        mqg.mqg_gcn_edge_weights(ctx, g, blocks, l, ew, sw)
        torch.cuda.synchronize()
        assert np.allclose(ew[:nnz].cpu().numpy(), ew_ref, rtol=1.2e-7, atol=0)
        assert np.allclose(sw[:nd].cpu().numpy(), sw_ref, rtol=1.2e-7, atol=0)
        assert torch.all(ew[nnz:] == -1.0) and torch.all(sw[nd:] == -1.0)
        # the whole estimator, GPU weights + GPU sum against oracle weights + oracle sum
        x = rng.standard_normal((ns, dim)).astype(np.float32)
        ref = oracle.weighted_aggregate(b["indptr"], b["indices"], ew_ref, sw_ref, x)
        xd = torch.zeros((blocks.bounds[l][1], dim), device="cuda")
        xd[:ns] = torch.from_numpy(x).cuda()
        out = torch.zeros((blocks.bounds[l][0], dim), device="cuda")
        mqg.mqg_weighted_aggregate(ctx, blocks, l, ew, sw, xd, out)
        torch.cuda.synchronize()
        check(out[:nd].cpu().numpy(), ref, row_mass(b["indptr"], ew_ref, sw_ref, x), 1e-5)
        # adjoint identity <M x, g> == <x, M^T g>, both sides on the GPU
        gd = torch.randn((blocks.bounds[l][0], dim), device="cuda")
        gx = torch.zeros((blocks.bounds[l][1], dim), device="cuda")
        mqg.mqg_weighted_aggregate_backward(ctx, blocks, l, ew, sw, gd, gx)
        torch.cuda.synchronize()
        lhs = float((out[:nd].double() * gd[:nd].double()).sum())
        rhs = float((xd[:ns].double() * gx[:ns].double()).sum())
        assert abs(lhs - rhs) < 1e-4 * max(1.0, abs(lhs))


def test_weighted_full_size_medium_block(mqg):
    """Block 0 of a "medium" mini-batch (252 k edges, 602 fp32 columns): weights of every edge, sums
    on sampled rows."""
    w = synth.WORKLOADS["medium"]
    rp, ci = synth.build_graph(w, seed=0, device="cuda")
    n = rp.numel() - 1
    g = mqg.Graph(rp, ci)
    fanouts = list(w.fanouts)
    ctx = mqg.Context(g, w.batch, fanouts)
    blocks = mqg.Blocks(g, w.batch, fanouts)
    seeds = synth.seed_batches(n, w.batch, 1, seed=2)[0]
    b = hip_sample(mqg, ctx, g, blocks, seeds, fanouts, 3)[0]
    nd, ns, nnz = b["num_dst"], b["num_src"], b["nnz"]
    rp_np = rp.cpu().numpy().astype(np.int64)
    ew_ref, sw_ref = oracle.gcn_edge_weights(rp_np, b["src_ids"], b["indptr"], b["indices"])
    ew = torch.zeros(blocks.bounds[0][2], device="cuda")
    sw = torch.zeros(blocks.bounds[0][0], device="cuda")
    mqg.mqg_gcn_edge_weights(ctx, g, blocks, 0, ew, sw)
    x = torch.randn((blocks.bounds[0][1], w.dim), device="cuda", generator=torch.Generator("cuda").manual_seed(1))
    out = torch.zeros((blocks.bounds[0][0], w.dim), device="cuda")
    mqg.mqg_weighted_aggregate(ctx, blocks, 0, ew, sw, x, out)
    gx = torch.zeros_like(x)
    mqg.mqg_weighted_aggregate_backward(ctx, blocks, 0, ew, sw, out, gx)
    torch.cuda.synchronize()
    assert np.allclose(ew[:nnz].cpu().numpy(), ew_ref, rtol=1.2e-7, atol=0)
    assert np.allclose(sw[:nd].cpu().numpy(), sw_ref, rtol=1.2e-7, atol=0)
    rng = np.random.default_rng(0)
    rows = np.unique(rng.integers(0, nd, 600))
    counts = (b["indptr"][rows + 1] - b["indptr"][rows]).astype(np.int64)
    sub_ptr = np.concatenate([[0], np.cumsum(counts)])
    sel = np.concatenate([np.arange(b["indptr"][r], b["indptr"][r + 1]) for r in rows])
    used, inv = np.unique(b["indices"][sel], return_inverse=True)
    x_sub = torch.cat([x[torch.from_numpy(rows).cuda()], x[torch.from_numpy(used.astype(np.int64)).cuda()]]).cpu().numpy()
    ref = oracle.weighted_aggregate(sub_ptr, (len(rows) + inv).astype(np.int32), ew_ref[sel], sw_ref[rows], x_sub)
    check(out[torch.from_numpy(rows).cuda()].cpu().numpy(), ref, row_mass(sub_ptr, ew_ref[sel], sw_ref[rows], x_sub), 1e-5)
    # backward on sampled sources: every edge into them, from the oracle's dense definition
    srcs = np.unique(np.concatenate([rng.integers(0, ns, 300), np.arange(5)]))
    out_np = out[:nd].cpu().numpy().astype(np.float64)
    dst_of_edge = np.repeat(np.arange(nd), np.diff(b["indptr"]))
    for s in srcs[:80]:
        e = np.nonzero(b["indices"] == s)[0]
        ref_row = (ew_ref[e][:, None] * out_np[dst_of_edge[e]]).sum(axis=0)
        mass = np.abs(ew_ref[e]).sum()
        if s < nd:
            ref_row = ref_row + sw_ref[s] * out_np[s]
            mass += abs(sw_ref[s])
        err = np.abs(gx[int(s)].cpu().numpy().astype(np.float64) - ref_row)
        assert np.all(err <= 1e-5 * np.maximum(np.abs(ref_row), mass * np.abs(out_np).mean())), int(s)


def test_weighted_argument_errors(mqg):
    ctx, blocks = bare_blocks(mqg, np.array([0, 1], dtype=np.int64), np.zeros(1, np.int32), 1, 1)
    x = torch.ones((1, 4), device="cuda")
    o = torch.ones((1, 4), device="cuda")
    ew = torch.ones(1, device="cuda")
    rc = mqg.lib.mqg_weighted_aggregate(ctx.h, blocks.c[0], None, None, x.data_ptr(), 4, o.data_ptr(), 4, 4, 0, None)
    assert rc == mqg.MQG_ERR_INVALID_ARG
    rc = mqg.lib.mqg_weighted_aggregate(ctx.h, blocks.c[0], ew.data_ptr(), None, x.data_ptr(), 2, o.data_ptr(), 4, 4, 0, None)
    assert rc == mqg.MQG_ERR_INVALID_ARG
    rc = mqg.lib.mqg_weighted_aggregate_backward(ctx.h, blocks.c[0], None, None, x.data_ptr(), 4, o.data_ptr(), 4, 4, 0, None)
    assert rc == mqg.MQG_ERR_INVALID_ARG
    rc = mqg.lib.mqg_weighted_aggregate_backward(ctx.h, blocks.c[0], ew.data_ptr(), None, x.data_ptr(), 4, o.data_ptr(), 4, 4, 9, None)
    assert rc == mqg.MQG_ERR_INVALID_ARG
    rc = mqg.lib.mqg_gcn_edge_weights(ctx.h, blocks._keep[3].c, blocks.c[0], ew.data_ptr(), None, None)
    assert rc == mqg.MQG_ERR_INVALID_ARG
