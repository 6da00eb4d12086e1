"""Seeded synthetic inputs: power-law graphs, node features and seed batches.

This module only manufactures inputs.  It contains none of the method's
arithmetic (no sampling keys, no dedup, no gather, no aggregation) and is the
one module that both the HIP path's tests and the CPU oracle's tests draw
their inputs from.  Everything is a deterministic function of the integer
seeds given, for a fixed device type.

The graphs stand in for the datasets of the paper's Table 1 (Reddit,
ogbn-products, ...), which are not available offline: Chung-Lu random graphs
with a power-law expected-degree sequence, made simple (no self loops, no
multi-edges), symmetrised, rows sorted ascending, node ids randomly permuted
so that degree is not monotone in id.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch


# --------------------------------------------------------------------------
# Chung-Lu power-law graph
# --------------------------------------------------------------------------

def _expected_degrees(num_nodes: int, total: float, gamma: float, cap: float) -> torch.Tensor:
    """w_i = c * (i + i0)^(-1/(gamma-1)), sum(w) = total, w_0 = cap (float64, CPU)."""
    alpha = 1.0 / (gamma - 1.0)
    idx = torch.arange(num_nodes, dtype=torch.float64)

    def w0_for(i0: float) -> float:
        s = torch.pow(idx + i0, -alpha).sum().item()
        return total * (i0 ** -alpha) / s

    lo, hi = 1e-3, float(num_nodes) * 64.0
    if w0_for(lo) <= cap:            # even the sharpest head stays below the cap
        i0 = lo
    else:
        for _ in range(80):          # w0 decreases monotonically in i0
            mid = math.sqrt(lo * hi)
            if w0_for(mid) > cap:
                lo = mid
            else:
                hi = mid
        i0 = hi
    w = torch.pow(idx + i0, -alpha)
    return w * (total / w.sum())


def chung_lu_graph(num_nodes: int, target_directed_edges: int, *, gamma: float = 2.1,
                   max_degree: Optional[float] = None, seed: int = 0,
                   device: str = "cpu", ptr_dtype=torch.int64, idx_dtype=torch.int64,
                   chunk: int = 1 << 26):
    """Return (row_ptr[N+1], col_idx[E]) of a simple symmetric Chung-Lu graph.

    Endpoints of target_directed_edges/2 undirected pairs are drawn with
    probability proportional to w_u * w_v; self loops and repeated pairs are
    dropped, so the realised edge count is somewhat below the target.
    """
    n = int(num_nodes)
    total = float(target_directed_edges)
    cap = float(max_degree) if max_degree is not None else math.sqrt(total)
    w = _expected_degrees(n, total, gamma, cap)
    cdf = torch.cumsum(w, 0)
    cdf = (cdf / cdf[-1]).to(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    perm = torch.randperm(n, generator=gen, device=device)
    pairs = int(target_directed_edges) // 2
    keys = []
    done = 0
    while done < pairs:
        m = min(chunk, pairs - done)
        u = torch.searchsorted(cdf, torch.rand(m, generator=gen, device=device, dtype=torch.float64))
        v = torch.searchsorted(cdf, torch.rand(m, generator=gen, device=device, dtype=torch.float64))
        u.clamp_(max=n - 1)
        v.clamp_(max=n - 1)
        u = perm[u]
        v = perm[v]
        keep = u != v
        u, v = u[keep], v[keep]
        lo, hi = torch.minimum(u, v), torch.maximum(u, v)
        keys.append(torch.unique(lo * n + hi))
        done += m
    und = torch.unique(torch.cat(keys)) if len(keys) > 1 else keys[0]
    del keys
    lo = und // n
    hi = und - lo * n
    del und
    both = torch.cat([lo * n + hi, hi * n + lo])
    del lo, hi
    both, _ = torch.sort(both)
    rows = both // n
    cols = (both - rows * n).to(idx_dtype)
    del both
    counts = torch.bincount(rows, minlength=n)
    del rows
    row_ptr = torch.zeros(n + 1, dtype=torch.int64, device=device)
    torch.cumsum(counts, 0, out=row_ptr[1:])
    return row_ptr.to(ptr_dtype), cols


# --------------------------------------------------------------------------
# Features and seed batches
# --------------------------------------------------------------------------

def node_features(num_nodes: int, dim: int, *, dtype=torch.float32, seed: int = 1,
                  device: str = "cpu", out: Optional[torch.Tensor] = None,
                  chunk_rows: int = 1 << 20) -> torch.Tensor:
    """N(0,1) features, generated chunk by chunk so a pinned host `out` of any
    size can be filled from a GPU generator without a second full copy."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    if out is None:
        out = torch.empty((num_nodes, dim), dtype=dtype, device=device)
    for r0 in range(0, num_nodes, chunk_rows):
        r1 = min(num_nodes, r0 + chunk_rows)
        blk = torch.randn((r1 - r0, dim), generator=gen, device=device, dtype=torch.float32)
        out[r0:r1, :dim].copy_(blk.to(dtype))
    return out


def aligned_row_stride(dim: int, dtype=torch.float32) -> int:
    """Row stride (in elements) used for feature rows, in pinned host memory and in HBM: rows start
    on 64-byte boundaries when that costs at most 2 % more memory, otherwise on 16-byte boundaries.
    A row that starts inside a cache line makes the host link carry the unused parts of its first
    and last line, and makes its first and last line partial writes in HBM."""
    elt = torch.empty((), dtype=dtype).element_size()
    row_bytes = dim * elt
    stride = (row_bytes + 63) // 64 * 64
    if stride > 1.02 * row_bytes:
        stride = (row_bytes + 15) // 16 * 16
    return stride // elt


def pinned_features(num_nodes: int, dim: int, *, dtype=torch.float32, seed: int = 1, device: str = "cpu") -> torch.Tensor:
    """node_features() into pinned host memory laid out with aligned_row_stride(); returns the
    [num_nodes, dim] view."""
    feats = torch.empty((num_nodes, aligned_row_stride(dim, dtype)), dtype=dtype).pin_memory()[:, :dim]
    return node_features(num_nodes, dim, dtype=dtype, seed=seed, device=device, out=feats)


def seed_batches(num_nodes: int, batch: int, num_batches: int, *, seed: int = 2,
                 train_fraction: Optional[float] = None, dtype=torch.int64) -> List[torch.Tensor]:
    """Batches of distinct seed nodes: consecutive slices of one random
    permutation of the training set (the whole node set, or a random
    `train_fraction` of it).  CPU tensors."""
    gen = torch.Generator()
    gen.manual_seed(int(seed))
    perm = torch.randperm(num_nodes, generator=gen)
    if train_fraction is not None:
        perm = perm[: max(batch, int(num_nodes * train_fraction))]
    out = []
    for b in range(num_batches):
        lo = (b * batch) % max(1, perm.numel() - batch + 1)
        out.append(perm[lo:lo + batch].to(dtype).contiguous())
    return out


# --------------------------------------------------------------------------
# The five workloads
# --------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    num_nodes: int
    target_edges: int
    gamma: float
    max_degree: Optional[float]
    ptr_dtype: torch.dtype
    idx_dtype: torch.dtype
    dim: int
    feat_dtype: torch.dtype
    fanouts: List[int]          # indexed by block: fanouts[L-1] expands the seeds
    batch: int
    cache_pct: Optional[int]    # None: every row lives in HBM, no host fallback
    train_fraction: Optional[float] = None
    num_batches: int = 16
    in_flight: int = 1
    cache_sweep: List[int] = field(default_factory=list)


WORKLOADS = {
    "tiny": Workload("tiny", 10_000, 200_000, 2.1, None, torch.int32, torch.int32,
                     64, torch.float32, [10, 5], 256, None),
    "medium": Workload("medium", 232_965, 114_000_000, 2.1, 20_000.0, torch.int64, torch.int64,
                       602, torch.float32, [25, 10], 1024, 30),
    "large": Workload("large", 2_449_029, 124_000_000, 2.1, None, torch.int64, torch.int64,
                      100, torch.float32, [15, 10, 5], 1024, 20),
    "xlarge": Workload("xlarge", 111_000_000, 1_600_000_000, 2.1, 40_000.0, torch.int64, torch.int64,
                       128, torch.float16, [15, 10, 5], 1024, 10, train_fraction=0.01),
    "stress": Workload("stress", 2_449_029, 124_000_000, 2.1, None, torch.int64, torch.int64,
                       256, torch.float16, [15, 10, 5], 8192, 20, in_flight=4,
                       cache_sweep=[5, 20, 50]),
}


def launch_in_flight(w: Workload) -> int:
    """Mini-batches kept in flight (contexts x streams) when a workload is timed or checked at full
    size: what the workload states ("stress": four), otherwise three."""
    return w.in_flight if w.in_flight > 1 else 3


def scaled(w: Workload, factor: float, name: Optional[str] = None) -> Workload:
    """The same workload shape with node and edge counts multiplied by `factor`
    (mean degree, fanouts, feature width and batch size unchanged)."""
    import dataclasses
    n = max(w.batch * 4, int(w.num_nodes * factor))
    e = max(n * 4, int(w.target_edges * factor))
    md = None if w.max_degree is None else min(w.max_degree, n / 4)
    return dataclasses.replace(w, name=name or f"{w.name}@{factor:g}", num_nodes=n,
                               target_edges=e, max_degree=md)


def build_graph(w: Workload, *, seed: int = 0, device: str = "cpu"):
    return chung_lu_graph(w.num_nodes, w.target_edges, gamma=w.gamma, max_degree=w.max_degree,
                          seed=seed, device=device, ptr_dtype=w.ptr_dtype, idx_dtype=w.idx_dtype)
