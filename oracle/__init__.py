"""CPU oracle (test infrastructure only).

Thin ctypes wrapper over ``mqg_oracle.c``: the plain single-threaded C
statement of cache build, L-hop neighbour sampling into bipartite blocks,
feature gather and mean aggregation.  Only the tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; it shares nothing with
the GPU implementation and never imports it.

Inputs and outputs are numpy arrays.  Node ids, offsets and counts are int64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mqg_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a few hundred lines of C; under a second)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized(out_dir: str) -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer, as a second library
    (for the test that runs the pins against it; load it by setting MQG_ORACLE_LIB)."""
    os.makedirs(out_dir, exist_ok=True)
    path = os.path.join(out_dir, "liboracle_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                           "-Wall", "-Wextra", "-o", path, _SRC, "-lm"])
    return path


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(os.environ.get("MQG_ORACLE_LIB") or build())
    i64, u64, i32, vp = ctypes.c_int64, ctypes.c_uint64, ctypes.c_int32, ctypes.c_void_p
    lib.orc_mix.restype = u64
    lib.orc_mix.argtypes = [u64]
    lib.orc_key.restype = u64
    lib.orc_key.argtypes = [u64, i64, i64, i64]
    lib.orc_build_cache.restype = ctypes.c_int
    lib.orc_build_cache.argtypes = [i64, vp, i64, vp, vp]
    lib.orc_fill_cache_rows.restype = None
    lib.orc_fill_cache_rows.argtypes = [vp, i64, vp, i64, i64, vp, i64]
    lib.orc_sample_row.restype = i64
    lib.orc_sample_row.argtypes = [u64, i64, i64, i64, i64, vp]
    lib.orc_sample_block.restype = i64
    lib.orc_sample_block.argtypes = [vp, vp, vp, i64, i64, i64, u64, i64, i64, vp, vp, vp, vp]
    lib.orc_sample_row_prioritised.restype = i64
    lib.orc_sample_row_prioritised.argtypes = [u64, i64, i64, i64, i64, vp, vp, vp]
    lib.orc_sample_block_prioritised.restype = i64
    lib.orc_sample_block_prioritised.argtypes = [vp, vp, vp, i64, i64, i64, u64, i64, i64, vp, vp, vp, vp, vp]
    lib.orc_gather.restype = None
    lib.orc_gather.argtypes = [vp, i64, vp, i64, vp, vp, i64, i64, vp, i64, vp, vp]
    lib.orc_half_to_double.restype = ctypes.c_double
    lib.orc_half_to_double.argtypes = [ctypes.c_uint16]
    lib.orc_float_to_half.restype = ctypes.c_uint16
    lib.orc_float_to_half.argtypes = [ctypes.c_float]
    lib.orc_mean_aggregate.restype = None
    lib.orc_mean_aggregate.argtypes = [vp, vp, i64, vp, i64, vp, i64, i64, ctypes.c_int]
    lib.orc_mean_aggregate_backward.restype = ctypes.c_int
    lib.orc_mean_aggregate_backward.argtypes = [vp, vp, i64, i64, vp, i64, vp, i64, i64, ctypes.c_int]
    lib.orc_gcn_edge_weights.restype = None
    lib.orc_gcn_edge_weights.argtypes = [vp, vp, vp, vp, i64, vp, vp]
    lib.orc_weighted_aggregate.restype = None
    lib.orc_weighted_aggregate.argtypes = [vp, vp, i64, vp, vp, vp, i64, vp, i64, i64, ctypes.c_int]
    lib.orc_weighted_aggregate_backward.restype = ctypes.c_int
    lib.orc_weighted_aggregate_backward.argtypes = [vp, vp, i64, i64, vp, vp, vp, i64, vp, i64, i64, ctypes.c_int]
    lib.orc_build_cache_sampled.restype = ctypes.c_int
    lib.orc_build_cache_sampled.argtypes = [i64, vp, i64, u64, vp, vp]
    lib.orc_random_walk_scores.restype = ctypes.c_int
    lib.orc_random_walk_scores.argtypes = [i64, vp, vp, vp, i64, vp, i64, i64, vp]
    lib.orc_build_cache_by_score.restype = ctypes.c_int
    lib.orc_build_cache_by_score.argtypes = [i64, vp, i64, vp, vp]
    lib.orc_ladies_probabilities.restype = None
    lib.orc_ladies_probabilities.argtypes = [vp, vp, i64, vp, i64, ctypes.c_int, vp]
    lib.orc_ladies_block.restype = i64
    lib.orc_ladies_block.argtypes = [vp, vp, i64, vp, i64, i64, i64, u64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, i64, i64, vp, vp, vp, vp, vp]
    lib.orc_debias_coefficients.restype = None
    lib.orc_debias_coefficients.argtypes = [vp, i64, i64, vp]
    lib.orc_exp_ticket.restype = u64
    lib.orc_exp_ticket.argtypes = [u64]
    lib.orc_exp_tickets.restype = None
    lib.orc_exp_tickets.argtypes = [u64, i64, i64, i64, vp]
    lib.orc_build_cache_drawn_by_score.restype = ctypes.c_int
    lib.orc_build_cache_drawn_by_score.argtypes = [i64, vp, i64, u64, vp, vp]
    _lib = lib
    return lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int64)


# ------------------------------------------------------------------ keys

def mix(z: int) -> int:
    return int(_load().orc_mix(ctypes.c_uint64(z & 0xFFFFFFFFFFFFFFFF)))


def key(rng_seed: int, layer: int, node: int, slot: int) -> int:
    return int(_load().orc_key(ctypes.c_uint64(rng_seed & 0xFFFFFFFFFFFFFFFF), layer, node, slot))


def sample_row(rng_seed: int, layer: int, node: int, degree: int, fanout: int) -> np.ndarray:
    out = np.empty(max(1, fanout), dtype=np.int64)
    c = _load().orc_sample_row(ctypes.c_uint64(rng_seed & 0xFFFFFFFFFFFFFFFF), layer, node,
                               degree, fanout, _p(out))
    return out[:c].copy()


# ----------------------------------------------------------------- cache

@dataclass
class Cache:
    cached_ids: np.ndarray      # int64[num_cached], slot order
    slot_of: np.ndarray         # int32[N], -1 when not cached
    cache_rows: Optional[np.ndarray] = None   # [num_cached, dim] copy of the cached feature rows


def build_cache(row_ptr, num_cached: int, feats: Optional[np.ndarray] = None) -> Cache:
    rp = _i64(row_ptr)
    n = rp.shape[0] - 1
    ids = np.empty(max(1, num_cached), dtype=np.int64)
    slot_of = np.empty(max(1, n), dtype=np.int32)
    rc = _load().orc_build_cache(n, _p(rp), num_cached, _p(ids), _p(slot_of))
    if rc != 0:
        raise ValueError(f"orc_build_cache failed ({rc})")
    ids = ids[:num_cached]
    slot_of = slot_of[:n]
    rows = None
    if feats is not None:
        assert feats.ndim == 2 and feats.strides[1] == feats.itemsize
        rows = np.zeros((num_cached, feats.shape[1]), dtype=feats.dtype)
        _load().orc_fill_cache_rows(_p(ids), num_cached, _p(feats), feats.strides[0],
                                    feats.shape[1] * feats.itemsize, _p(rows),
                                    rows.strides[0] if num_cached else 0)
    return Cache(ids, slot_of, rows)


def _finish_cache(ids, slot_of, num_cached, n, feats):
    ids, slot_of = ids[:num_cached], slot_of[:n]
    rows = None
    if feats is not None:
        rows = np.zeros((num_cached, feats.shape[1]), dtype=feats.dtype)
        _load().orc_fill_cache_rows(_p(ids), num_cached, _p(feats), feats.strides[0],
                                    feats.shape[1] * feats.itemsize, _p(rows), rows.strides[0] if num_cached else 0)
    return Cache(ids, slot_of, rows)


def build_cache_sampled(row_ptr, num_cached: int, seed: int, feats: Optional[np.ndarray] = None) -> Cache:
    """Membership drawn with probability proportional to degree, without replacement (Eq. 13)."""
    rp = _i64(row_ptr)
    n = rp.shape[0] - 1
    ids = np.empty(max(1, num_cached), dtype=np.int64)
    slot_of = np.empty(max(1, n), dtype=np.int32)
    rc = _load().orc_build_cache_sampled(n, _p(rp), num_cached, ctypes.c_uint64(seed & 0xFFFFFFFFFFFFFFFF),
                                         _p(ids), _p(slot_of))
    if rc != 0:
        raise ValueError(f"orc_build_cache_sampled failed ({rc})")
    return _finish_cache(ids, slot_of, num_cached, n, feats)


WALK_PUSH, WALK_PRINTED = 0, 1


def random_walk_scores(row_ptr, col_idx, train_ids, step_fanouts: Sequence[int], form: int = WALK_PUSH) -> np.ndarray:
    """P^(L) of Eq. 14-15; step_fanouts[l-1] is the fanout of walk step l.  form: WALK_PUSH moves mass
    from a node to the nodes it samples from, (D A + I)^T P; WALK_PRINTED is (D A + I) P as printed."""
    rp, ci, tr = _i64(row_ptr), _i64(col_idx), _i64(train_ids)
    fo = _i64(list(step_fanouts))
    n = rp.shape[0] - 1
    out = np.zeros(max(1, n), dtype=np.float64)
    rc = _load().orc_random_walk_scores(n, _p(rp), _p(ci), _p(tr), tr.shape[0], _p(fo), fo.shape[0], form, _p(out))
    if rc != 0:
        raise ValueError(f"orc_random_walk_scores failed ({rc})")
    return out[:n]


def build_cache_by_score(scores: np.ndarray, num_cached: int, feats: Optional[np.ndarray] = None) -> Cache:
    sc = np.ascontiguousarray(scores, dtype=np.float64)
    n = sc.shape[0]
    ids = np.empty(max(1, num_cached), dtype=np.int64)
    slot_of = np.empty(max(1, n), dtype=np.int32)
    rc = _load().orc_build_cache_by_score(n, _p(sc), num_cached, _p(ids), _p(slot_of))
    if rc != 0:
        raise ValueError(f"orc_build_cache_by_score failed ({rc})")
    return _finish_cache(ids, slot_of, num_cached, n, feats)


def exp_ticket(r: int) -> int:
    return int(_load().orc_exp_ticket(ctypes.c_uint64(r & 0xFFFFFFFFFFFFFFFF)))


def exp_tickets(seed: int, layer: int, first: int, n: int) -> np.ndarray:
    """exp_ticket(key(seed, layer, first + i, 0)) for i in [0, n), as uint64."""
    out = np.zeros(max(1, n), dtype=np.uint64)
    _load().orc_exp_tickets(ctypes.c_uint64(seed & 0xFFFFFFFFFFFFFFFF), layer, first, n, _p(out))
    return out[:n]


def build_cache_drawn_by_score(scores: np.ndarray, num_cached: int, seed: int,
                               feats: Optional[np.ndarray] = None) -> Cache:
    """Membership drawn with probability proportional to the score, without replacement."""
    sc = np.ascontiguousarray(scores, dtype=np.float64)
    n = sc.shape[0]
    ids = np.empty(max(1, num_cached), dtype=np.int64)
    slot_of = np.empty(max(1, n), dtype=np.int32)
    rc = _load().orc_build_cache_drawn_by_score(n, _p(sc), num_cached, ctypes.c_uint64(seed), _p(ids), _p(slot_of))
    if rc != 0:
        raise ValueError(f"orc_build_cache_drawn_by_score failed ({rc})")
    return _finish_cache(ids, slot_of, num_cached, n, feats)


# -------------------------------------------------------------- sampling

@dataclass
class Block:
    num_dst: int
    src_ids: np.ndarray     # int64[num_src]; src_ids[:num_dst] are the destination nodes
    indptr: np.ndarray      # int64[num_dst+1]
    indices: np.ndarray     # int32[nnz], positions in src_ids
    nbr_global: np.ndarray  # int64[nnz], global ids of the sampled neighbours

    @property
    def num_src(self) -> int:
        return int(self.src_ids.shape[0])

    @property
    def nnz(self) -> int:
        return int(self.indices.shape[0])


def sample_row_prioritised(rng_seed: int, layer: int, node: int, nbrs, fanout: int, slot_of) -> np.ndarray:
    nb = _i64(nbrs)
    so = np.ascontiguousarray(slot_of, dtype=np.int32)
    out = np.empty(max(1, fanout), dtype=np.int64)
    c = _load().orc_sample_row_prioritised(ctypes.c_uint64(rng_seed & 0xFFFFFFFFFFFFFFFF), layer, node,
                                           nb.shape[0], fanout, _p(nb), _p(so), _p(out))
    return out[:c].copy()


def sample_blocks(row_ptr, col_idx, seeds, fanouts: Sequence[int], rng_seed: int, prio_slot_of=None) -> List[Block]:
    """blocks[l] feeds GNN layer l; blocks[L-1] has the seeds as destinations and
    uses fanouts[L-1]; the destinations of blocks[l-1] are the sources of blocks[l].
    prio_slot_of (int32[N], >= 0 for cached nodes): cached neighbours are drawn first."""
    rp, ci, dst = _i64(row_ptr), _i64(col_idx), _i64(seeds)
    prio = None if prio_slot_of is None else np.ascontiguousarray(prio_slot_of, dtype=np.int32)
    n = rp.shape[0] - 1
    L = len(fanouts)
    blocks: List[Optional[Block]] = [None] * L
    lib = _load()
    for l in range(L - 1, -1, -1):
        k = int(fanouts[l])
        nd = dst.shape[0]
        cap_nnz = nd * k
        cap_src = min(n, nd + cap_nnz) if n > 0 else nd
        cap_src = max(cap_src, nd)
        indptr = np.empty(nd + 1, dtype=np.int64)
        nbr = np.empty(max(1, cap_nnz), dtype=np.int64)
        src = np.empty(max(1, cap_src), dtype=np.int64)
        idx = np.empty(max(1, cap_nnz), dtype=np.int32)
        if prio is None:
            ns = lib.orc_sample_block(_p(rp), _p(ci), _p(dst), nd, k, l,
                                      ctypes.c_uint64(rng_seed & 0xFFFFFFFFFFFFFFFF), cap_nnz, cap_src,
                                      _p(indptr), _p(nbr), _p(src), _p(idx))
        else:
            ns = lib.orc_sample_block_prioritised(_p(rp), _p(ci), _p(dst), nd, k, l,
                                                  ctypes.c_uint64(rng_seed & 0xFFFFFFFFFFFFFFFF), cap_nnz, cap_src,
                                                  _p(indptr), _p(nbr), _p(src), _p(idx), _p(prio))
        if ns < 0:
            raise RuntimeError(f"orc_sample_block failed ({ns})")
        nnz = int(indptr[nd])
        blocks[l] = Block(nd, src[:ns].copy(), indptr, idx[:nnz].copy(), nbr[:nnz].copy())
        dst = blocks[l].src_ids
    return blocks  # type: ignore[return-value]


@dataclass
class WeightedBlock:
    num_dst: int
    src_ids: np.ndarray     # int64[num_src], ascending: the next layer's rows
    indptr: np.ndarray      # int64[num_dst+1]
    indices: np.ndarray     # int32[nnz], positions in src_ids
    edge_w: np.ndarray      # float64[nnz]
    mass: Optional[np.ndarray] = None

    @property
    def num_src(self) -> int:
        return int(self.src_ids.shape[0])

    @property
    def nnz(self) -> int:
        return int(self.indices.shape[0])


def debias_coefficients(p_drawn, population: int) -> np.ndarray:
    """Eq. 12: coefficients of the items drawn without replacement, in draw order."""
    p = np.ascontiguousarray(p_drawn, dtype=np.float64)
    beta = np.zeros(max(1, p.shape[0]), dtype=np.float64)
    _load().orc_debias_coefficients(_p(p), p.shape[0], population, _p(beta))
    return beta[:p.shape[0]]


def ladies_probabilities(row_ptr, col_idx, dst=None, flat: bool = False) -> np.ndarray:
    """Eq. 7 for the rows dst; dst=None: all rows (FastGCN's batch-independent probabilities);
    flat: proportional to the column norm instead of its square (Eq. 10)."""
    rp, ci = _i64(row_ptr), _i64(col_idx)
    n = rp.shape[0] - 1
    p = np.zeros(max(n, 1), dtype=np.float64)
    if dst is None:
        _load().orc_ladies_probabilities(_p(rp), _p(ci), n, None, 0, 1 if flat else 0, _p(p))
    else:
        d = _i64(dst)
        _load().orc_ladies_probabilities(_p(rp), _p(ci), n, _p(d), d.shape[0], 1 if flat else 0, _p(p))
    return p[:n]


def ladies_blocks(row_ptr, col_idx, seeds, layer_sizes: Sequence[int], rng_seed: int, normalise: bool = True,
                  want_mass: bool = False, fastgcn: bool = False, debias: bool = False, flat: bool = False) -> List[WeightedBlock]:
    """LADIES mini-batch: blocks[L-1] has the seeds as rows; layer_sizes[l] nodes are drawn as the
    sources of blocks[l], which are the rows of blocks[l-1]."""
    rp, ci, dst = _i64(row_ptr), _i64(col_idx), _i64(seeds)
    n = rp.shape[0] - 1
    L = len(layer_sizes)
    out: List[Optional[WeightedBlock]] = [None] * L
    lib = _load()
    for l in range(L - 1, -1, -1):
        s = int(layer_sizes[l])
        nd = dst.shape[0]
        cap_src = max(1, min(n, s))
        cap_nnz = max(1, nd * cap_src)
        src = np.empty(cap_src, dtype=np.int64)
        indptr = np.empty(nd + 1, dtype=np.int64)
        idx = np.empty(cap_nnz, dtype=np.int32)
        ew = np.empty(cap_nnz, dtype=np.float64)
        mass = np.zeros(max(n, 1), dtype=np.uint64) if want_mass else None
        ns = lib.orc_ladies_block(_p(rp), _p(ci), n, _p(dst), nd, s, l, ctypes.c_uint64(rng_seed & 0xFFFFFFFFFFFFFFFF),
                                  1 if normalise else 0, 1 if fastgcn else 0, 1 if debias else 0, 1 if flat else 0, cap_src, cap_nnz,
                                  _p(src), _p(indptr),
                                  _p(idx), _p(ew),
                                  None if mass is None else _p(mass))
        if ns < 0:
            raise RuntimeError(f"orc_ladies_block failed ({ns})")
        nnz = int(indptr[nd])
        out[l] = WeightedBlock(nd, src[:ns].copy(), indptr, idx[:nnz].copy(), ew[:nnz].copy(), mass)
        dst = out[l].src_ids
    return out  # type: ignore[return-value]


# ---------------------------------------------------------------- gather

def gather(ids, feats: np.ndarray, cache: Optional[Cache] = None):
    """Return (rows[len(ids), dim], hits, misses)."""
    ids = _i64(ids)
    assert feats.ndim == 2 and feats.strides[1] == feats.itemsize
    out = np.zeros((ids.shape[0], feats.shape[1]), dtype=feats.dtype)
    hits, misses = ctypes.c_int64(0), ctypes.c_int64(0)
    slot_of = rows = None
    cstride = 0
    if cache is not None:
        slot_of = np.ascontiguousarray(cache.slot_of, dtype=np.int32)
        rows = cache.cache_rows
        assert rows is not None
        cstride = rows.strides[0] if rows.shape[0] else 0
    _load().orc_gather(_p(ids), ids.shape[0], _p(feats), feats.strides[0], _p(slot_of), _p(rows),
                       cstride, feats.shape[1] * feats.itemsize, _p(out),
                       out.strides[0] if ids.shape[0] else 0, ctypes.byref(hits),
                       ctypes.byref(misses))
    return out, int(hits.value), int(misses.value)


# ------------------------------------------------------------- aggregate

def mean_aggregate(indptr, indices, x: np.ndarray) -> np.ndarray:
    """x: [num_src, dim] float32 or float16; returns [num_dst, dim] of the same dtype."""
    ip = _i64(indptr)
    ix = np.ascontiguousarray(np.asarray(indices), dtype=np.int32)
    assert x.dtype in (np.float32, np.float16) and x.ndim == 2
    x = np.ascontiguousarray(x)
    nd = ip.shape[0] - 1
    out = np.zeros((nd, x.shape[1]), dtype=x.dtype)
    _load().orc_mean_aggregate(_p(ip), _p(ix), nd, _p(x), x.shape[1], _p(out), x.shape[1],
                               x.shape[1], 1 if x.dtype == np.float16 else 0)
    return out


def mean_aggregate_backward(indptr, indices, num_src: int, grad_out: np.ndarray) -> np.ndarray:
    """grad_out: [num_dst, dim] float32 or float16; returns grad_x [num_src, dim], same dtype."""
    ip = _i64(indptr)
    ix = np.ascontiguousarray(np.asarray(indices), dtype=np.int32)
    assert grad_out.dtype in (np.float32, np.float16) and grad_out.ndim == 2
    g = np.ascontiguousarray(grad_out)
    nd = ip.shape[0] - 1
    assert g.shape[0] >= nd
    out = np.zeros((num_src, g.shape[1]), dtype=g.dtype)
    rc = _load().orc_mean_aggregate_backward(_p(ip), _p(ix), nd, num_src, _p(g), g.shape[1], _p(out),
                                             g.shape[1], g.shape[1], 1 if g.dtype == np.float16 else 0)
    if rc != 0:
        raise MemoryError("orc_mean_aggregate_backward")
    return out


def gcn_edge_weights(row_ptr, src_ids, indptr, indices):
    """Weights of the sampled estimator of P H (Eq. 1-3) for one block.
    Returns (edge_w [nnz] float64, self_w [num_dst] float64)."""
    rp, sid, ip = _i64(row_ptr), _i64(src_ids), _i64(indptr)
    ix = np.ascontiguousarray(np.asarray(indices), dtype=np.int32)
    nd = ip.shape[0] - 1
    ew = np.zeros(max(int(ip[-1]), 1), dtype=np.float64)
    sw = np.zeros(max(nd, 1), dtype=np.float64)
    _load().orc_gcn_edge_weights(_p(rp), _p(sid), _p(ip), _p(ix), nd, _p(ew), _p(sw))
    return ew[:int(ip[-1])], sw[:nd]


def weighted_aggregate(indptr, indices, edge_w, self_w, x: np.ndarray) -> np.ndarray:
    """out[i] = self_w[i] x[i] + sum_p edge_w[p] x[indices[p]]; self_w may be None."""
    ip = _i64(indptr)
    ix = np.ascontiguousarray(np.asarray(indices), dtype=np.int32)
    ew = np.ascontiguousarray(np.asarray(edge_w), dtype=np.float64)
    sw = None if self_w is None else np.ascontiguousarray(np.asarray(self_w), dtype=np.float64)
    assert x.dtype in (np.float32, np.float16) and x.ndim == 2
    x = np.ascontiguousarray(x)
    nd = ip.shape[0] - 1
    out = np.zeros((nd, x.shape[1]), dtype=x.dtype)
    _load().orc_weighted_aggregate(_p(ip), _p(ix), nd, _p(ew), None if sw is None else _p(sw), _p(x), x.shape[1],
                                   _p(out), x.shape[1], x.shape[1], 1 if x.dtype == np.float16 else 0)
    return out


def weighted_aggregate_backward(indptr, indices, num_src: int, edge_w, self_w, grad_out: np.ndarray) -> np.ndarray:
    ip = _i64(indptr)
    ix = np.ascontiguousarray(np.asarray(indices), dtype=np.int32)
    ew = np.ascontiguousarray(np.asarray(edge_w), dtype=np.float64)
    sw = None if self_w is None else np.ascontiguousarray(np.asarray(self_w), dtype=np.float64)
    g = np.ascontiguousarray(grad_out)
    assert g.dtype in (np.float32, np.float16) and g.ndim == 2
    nd = ip.shape[0] - 1
    out = np.zeros((num_src, g.shape[1]), dtype=g.dtype)
    rc = _load().orc_weighted_aggregate_backward(_p(ip), _p(ix), nd, num_src, _p(ew), None if sw is None else _p(sw),
                                                 _p(g), g.shape[1], _p(out), g.shape[1], g.shape[1],
                                                 1 if g.dtype == np.float16 else 0)
    if rc != 0:
        raise MemoryError("orc_weighted_aggregate_backward")
    return out


def queue_size(max_prepare_ms: float, mean_compute_ms: float, total_mem_bytes: int, peak_mem_bytes: int,
               margin_percent: int, mem_per_batch_bytes: int):
    """Queue depth of the paper's Sec. IV "Determining Optimal Queue Size" (Eq. 22, 23), written out:
    C = floor(M_Q / M_batch) with M_Q = total - peak*(1 + margin/100) (exact rational arithmetic),
    Q = min(C, max(2, ceil(max_prepare / mean_compute))).  Returns (Q, C)."""
    import math
    from fractions import Fraction
    m_q = Fraction(total_mem_bytes) - Fraction(peak_mem_bytes) * (1 + Fraction(margin_percent, 100))
    cap = math.floor(m_q / mem_per_batch_bytes)
    want = max(2, math.ceil(max_prepare_ms / mean_compute_ms))
    return min(cap, want), cap


def half_to_double(bits: int) -> float:
    return float(_load().orc_half_to_double(ctypes.c_uint16(bits)))


def float_to_half(f: float) -> int:
    return int(_load().orc_float_to_half(ctypes.c_float(f)))
