"""ctypes binding of libmqg.so - argument marshalling only.

The four operations keep the names of the C ABI (``include/mqg.h``):
``mqg_build_cache``, ``mqg_sample_blocks``, ``mqg_gather_features`` and
``mqg_sage_mean_aggregate``.  Torch is used for device memory, pinned host
memory and streams; every step of the path runs in the library's kernels.
There is no fallback: if the shared library is missing, importing this module
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmqg.so")

MQG_OK, MQG_ERR_INVALID_ARG, MQG_ERR_CAPACITY, MQG_ERR_HIP, MQG_ERR_UNSUPPORTED = 0, -1, -2, -3, -4
MQG_F32, MQG_F16 = 0, 1
MQG_I32, MQG_I64 = 0, 1
MQG_OPT_FORCE_SLOW_SELECT, MQG_OPT_PROFILE, MQG_OPT_MISS_INFLIGHT_BYTES, MQG_OPT_HEAVY_DEGREE, MQG_OPT_DEDUP_HASH = 1, 2, 3, 4, 5
MQG_OPT_LAYERWISE_CANDIDATES = 6
MQG_MAX_FANOUT, MQG_MAX_LAYERS = 64, 8
MQG_CACHE_TOP_DEGREE, MQG_CACHE_DEGREE_SAMPLED, MQG_CACHE_RANDOM_WALK, MQG_CACHE_RANDOM_WALK_SAMPLED = 0, 1, 2, 3
MQG_WALK_PUSH, MQG_WALK_PRINTED = 0, 1

EXPORTS = [
    "mqg_version", "mqg_ctx_create", "mqg_ctx_destroy", "mqg_last_error", "mqg_ctx_set_option",
    "mqg_ctx_kernel_time", "mqg_ctx_reset_profile", "mqg_ctx_kernel_names", "mqg_build_cache",
    "mqg_sample_blocks", "mqg_gather_features", "mqg_sage_mean_aggregate", "mqg_sage_mean_aggregate_backward",
    "mqg_queue_size", "mqg_build_cache_ex", "mqg_gcn_edge_weights", "mqg_weighted_aggregate",
    "mqg_weighted_aggregate_backward", "mqg_ctx_set_sampling_priority", "mqg_sample_layerwise",
    "mqg_select_smallest_keys", "mqg_select_row_candidates", "mqg_sample_blocks_seed_dev",
    "mqg_gather_features_static", "mqg_exp_tickets", "mqg_gather_features_cached", "mqg_gather_features_missed",
    "mqg_ctx_reserve",
]

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_04707_amd.build` "
                      "(hipcc, gfx950).  There is no CPU fallback.")

lib = ctypes.CDLL(LIB_PATH)

_i64, _i32, _vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p


class CGraph(ctypes.Structure):
    _fields_ = [("num_nodes", _i64), ("num_edges", _i64), ("ptr_type", _i32), ("idx_type", _i32),
                ("row_ptr", _vp), ("col_idx", _vp)]


class CCache(ctypes.Structure):
    _fields_ = [("num_nodes", _i64), ("num_cached", _i64), ("dim", _i32), ("dtype", _i32),
                ("feats", _vp), ("feat_stride", _i64), ("cache_rows", _vp), ("cache_stride", _i64),
                ("slot_of", _vp), ("cached_ids", _vp)]


class CBlock(ctypes.Structure):
    _fields_ = [("cap_dst", _i64), ("cap_src", _i64), ("cap_nnz", _i64), ("src_ids", _vp),
                ("indptr", _vp), ("indices", _vp), ("sizes", _vp)]


class CCachePlan(ctypes.Structure):
    _fields_ = [("policy", _i32), ("num_steps", _i32), ("seed", ctypes.c_uint64), ("train_ids", _vp),
                ("num_train", _i64), ("step_fanouts", ctypes.POINTER(_i32)), ("scores_out", _vp),
                ("walk_form", _i32), ("graph_symmetric", _i32)]


lib.mqg_version.restype = _i32
lib.mqg_version.argtypes = []
lib.mqg_ctx_create.restype = ctypes.c_int
lib.mqg_ctx_create.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(CGraph), _i32, ctypes.POINTER(_i32), _i32]
lib.mqg_ctx_destroy.restype = ctypes.c_int
lib.mqg_ctx_destroy.argtypes = [_vp]
lib.mqg_last_error.restype = ctypes.c_char_p
lib.mqg_last_error.argtypes = [_vp]
lib.mqg_ctx_set_option.restype = ctypes.c_int
lib.mqg_ctx_set_option.argtypes = [_vp, _i32, _i64]
lib.mqg_ctx_reserve.restype = ctypes.c_int
lib.mqg_ctx_reserve.argtypes = [_vp, _i32, _i64]
MQG_RESERVE_BACKWARD, MQG_RESERVE_LAYERWISE, MQG_RESERVE_DEDUP_HASH, MQG_RESERVE_SAMPLING_PRIORITY, MQG_RESERVE_CACHE_BUILD = 1, 2, 4, 8, 16
lib.mqg_ctx_kernel_time.restype = ctypes.c_int
lib.mqg_ctx_kernel_time.argtypes = [_vp, ctypes.c_char_p, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_i64)]
lib.mqg_ctx_reset_profile.restype = ctypes.c_int
lib.mqg_ctx_reset_profile.argtypes = [_vp]
lib.mqg_ctx_kernel_names.restype = ctypes.c_int
lib.mqg_ctx_kernel_names.argtypes = [_vp, ctypes.c_char_p, _i64]
lib.mqg_build_cache.restype = ctypes.c_int
lib.mqg_build_cache.argtypes = [_vp, ctypes.POINTER(CGraph), ctypes.POINTER(CCache), _vp]
lib.mqg_build_cache_ex.restype = ctypes.c_int
lib.mqg_build_cache_ex.argtypes = [_vp, ctypes.POINTER(CGraph), ctypes.POINTER(CCache), ctypes.POINTER(CCachePlan), _vp]
lib.mqg_sample_blocks.restype = ctypes.c_int
lib.mqg_sample_blocks.argtypes = [_vp, ctypes.POINTER(CGraph), _vp, _i32, ctypes.POINTER(_i32), _i32,
                                  ctypes.c_uint64, ctypes.POINTER(CBlock), _vp]
lib.mqg_gather_features.restype = ctypes.c_int
lib.mqg_gather_features.argtypes = [_vp, ctypes.POINTER(CCache), _i32, _vp, _vp, _i64, _vp, _i64, _vp, _vp]
for _name in ("mqg_gather_features_cached", "mqg_gather_features_missed"):
    getattr(lib, _name).restype = ctypes.c_int
    getattr(lib, _name).argtypes = [_vp, ctypes.POINTER(CCache), _i32, _vp, _vp, _i64, _vp, _i64, _vp, _vp]
lib.mqg_gather_features_static.restype = ctypes.c_int
lib.mqg_gather_features_static.argtypes = [ctypes.POINTER(CCache), _i32, _vp, _vp, _i64, _vp, _i64, _vp, _vp]
MQG_GATHER_STATIC_MAX_IDS = 1 << 20
lib.mqg_sage_mean_aggregate.restype = ctypes.c_int
lib.mqg_sage_mean_aggregate.argtypes = [_vp, ctypes.POINTER(CBlock), _vp, _i64, _vp, _i64, _i32, _i32, _vp]
lib.mqg_sage_mean_aggregate_backward.restype = ctypes.c_int
lib.mqg_sage_mean_aggregate_backward.argtypes = [_vp, ctypes.POINTER(CBlock), _vp, _i64, _vp, _i64, _i32, _i32, _vp]
lib.mqg_queue_size.restype = ctypes.c_int
lib.mqg_gcn_edge_weights.restype = ctypes.c_int
lib.mqg_gcn_edge_weights.argtypes = [_vp, ctypes.POINTER(CGraph), ctypes.POINTER(CBlock), _vp, _vp, _vp]
lib.mqg_weighted_aggregate.restype = ctypes.c_int
lib.mqg_weighted_aggregate.argtypes = [_vp, ctypes.POINTER(CBlock), _vp, _vp, _vp, _i64, _vp, _i64, _i32, _i32, _vp]
lib.mqg_weighted_aggregate_backward.restype = ctypes.c_int
lib.mqg_weighted_aggregate_backward.argtypes = [_vp, ctypes.POINTER(CBlock), _vp, _vp, _vp, _i64, _vp, _i64, _i32, _i32, _vp]
lib.mqg_ctx_set_sampling_priority.restype = ctypes.c_int
lib.mqg_ctx_set_sampling_priority.argtypes = [_vp, ctypes.POINTER(CGraph), ctypes.POINTER(CCache), _vp]
lib.mqg_sample_layerwise.restype = ctypes.c_int
lib.mqg_sample_layerwise.argtypes = [_vp, ctypes.POINTER(CGraph), _vp, _i32, ctypes.POINTER(_i32), _i32, ctypes.c_uint64,
                                     _i32, _i32, ctypes.POINTER(CBlock), ctypes.POINTER(_vp), _vp]
MQG_LAYERWISE_LADIES, MQG_LAYERWISE_FASTGCN, MQG_LAYERWISE_DEBIAS, MQG_LAYERWISE_FLAT = 0, 1, 2, 4
lib.mqg_select_smallest_keys.restype = ctypes.c_int
lib.mqg_select_smallest_keys.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp]
lib.mqg_select_row_candidates.restype = ctypes.c_int
lib.mqg_select_row_candidates.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp]
lib.mqg_exp_tickets.restype = ctypes.c_int
lib.mqg_exp_tickets.argtypes = [_vp, ctypes.c_uint64, _i64, _i64, _i64, _vp, _vp]
lib.mqg_sample_blocks_seed_dev.restype = ctypes.c_int
lib.mqg_sample_blocks_seed_dev.argtypes = [_vp, ctypes.POINTER(CGraph), _vp, _i32, ctypes.POINTER(_i32), _i32, _vp,
                                           ctypes.POINTER(CBlock), _vp]
lib.mqg_queue_size.argtypes = [ctypes.c_double, ctypes.c_double, _i64, _i64, _i32, _i64, ctypes.POINTER(_i64),
                               ctypes.POINTER(_i64)]


class MqgError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"mqg error {code}: {msg}")
        self.code = code


def _itype(t: torch.Tensor) -> int:
    if t.dtype == torch.int32:
        return MQG_I32
    if t.dtype == torch.int64:
        return MQG_I64
    raise TypeError(f"index tensors must be int32 or int64, got {t.dtype}")


def _dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MQG_F32
    if t.dtype == torch.float16:
        return MQG_F16
    raise TypeError(f"features must be float32 or float16, got {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


class Graph:
    """CSR graph resident on the GPU (the tensors are kept alive here)."""

    def __init__(self, row_ptr: torch.Tensor, col_idx: torch.Tensor):
        assert row_ptr.is_cuda and col_idx.is_cuda and row_ptr.is_contiguous() and col_idx.is_contiguous()
        self.row_ptr, self.col_idx = row_ptr, col_idx
        self.num_nodes = row_ptr.numel() - 1
        self.c = CGraph(self.num_nodes, col_idx.numel(), _itype(row_ptr), _itype(col_idx),
                        row_ptr.data_ptr(), col_idx.data_ptr())

    @property
    def idx_dtype(self):
        return self.col_idx.dtype


class Context:
    def __init__(self, graph: Graph, max_seeds: int, max_fanouts: Sequence[int]):
        self.graph = graph
        self.max_fanouts = list(max_fanouts)
        self.max_seeds = int(max_seeds)
        h = _vp()
        arr = (_i32 * len(max_fanouts))(*max_fanouts)
        rc = lib.mqg_ctx_create(ctypes.byref(h), ctypes.byref(graph.c), max_seeds, arr, len(max_fanouts))
        if rc != MQG_OK:
            raise MqgError(rc, lib.mqg_last_error(None).decode())
        self.h = h

    def check(self, rc: int):
        if rc != MQG_OK:
            raise MqgError(rc, lib.mqg_last_error(self.h).decode())

    def set_option(self, option: int, value: int):
        self.check(lib.mqg_ctx_set_option(self.h, option, value))

    def reserve(self, what: int, layerwise_rows: int = 0):
        """Allocate optional-path scratch now (a sum of MQG_RESERVE_*)."""
        self.check(lib.mqg_ctx_reserve(self.h, what, layerwise_rows))

    def set_sampling_priority(self, cache, stream=None):
        """Draw cached neighbours first (cache: a Cache, or None for the uniform draw)."""
        self.check(lib.mqg_ctx_set_sampling_priority(self.h, ctypes.byref(self.graph.c),
                                                     ctypes.byref(cache.c) if cache is not None else None,
                                                     _stream(stream)))

    def kernel_time(self, name: str):
        ms, n = ctypes.c_double(0), _i64(0)
        self.check(lib.mqg_ctx_kernel_time(self.h, name.encode(), ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def kernel_names(self) -> List[str]:
        buf = ctypes.create_string_buffer(8192)
        self.check(lib.mqg_ctx_kernel_names(self.h, buf, 8192))
        return [s for s in buf.value.decode().split("\n") if s]

    def reset_profile(self):
        self.check(lib.mqg_ctx_reset_profile(self.h))

    def close(self):
        if getattr(self, "h", None):
            lib.mqg_ctx_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def block_bounds(num_nodes: int, num_seeds: int, fanouts: Sequence[int]):
    """Worst-case (cap_dst, cap_src, cap_nnz) per block, the bounds the library checks."""
    L = len(fanouts)
    out = [None] * L
    dst = num_seeds
    for l in range(L - 1, -1, -1):
        nnz = dst * fanouts[l]
        src = max(dst, min(num_nodes, dst + nnz))
        out[l] = (dst, src, nnz)
        dst = src
    return out


class Blocks:
    """Device buffers of the L blocks of one mini-batch, sized by the worst-case bounds."""

    def __init__(self, graph: Graph, max_seeds: int, fanouts: Sequence[int], device=None):
        device = device or graph.col_idx.device
        self.fanouts = list(fanouts)
        self.L = len(fanouts)
        self.bounds = block_bounds(graph.num_nodes, max_seeds, fanouts)
        self.src_ids, self.indptr, self.indices = [], [], []
        self.sizes = torch.zeros((self.L, 4), dtype=torch.int64, device=device)
        self.c = (CBlock * self.L)()
        for l, (cd, cs, cn) in enumerate(self.bounds):
            self.src_ids.append(torch.empty(max(cs, 1), dtype=graph.idx_dtype, device=device))
            self.indptr.append(torch.empty(cd + 1, dtype=torch.int32, device=device))
            self.indices.append(torch.empty(max(cn, 1), dtype=torch.int32, device=device))
            self.c[l] = CBlock(cd, cs, cn, self.src_ids[l].data_ptr(), self.indptr[l].data_ptr(),
                               self.indices[l].data_ptr(), self.sizes[l].data_ptr())

    def host_sizes(self):
        """[(num_dst, num_src, nnz, flags)] - synchronises."""
        return [tuple(int(x) for x in row) for row in self.sizes.cpu().tolist()]


class LayerwiseBlocks(Blocks):
    """Buffers of the L weighted blocks of one layer-wise mini-batch: rows of block L-1 = the seeds,
    sources of block l = the layer_sizes[l] drawn nodes = the rows of block l-1."""

    def __init__(self, graph: Graph, max_seeds: int, layer_sizes: Sequence[int], nnz_per_row: Optional[int] = None,
                 device=None):
        device = device or graph.col_idx.device
        self.layer_sizes = list(layer_sizes)
        self.L = len(layer_sizes)
        n = graph.num_nodes
        self.bounds = []
        rows = max_seeds
        for l in range(self.L - 1, -1, -1):
            src = min(n, layer_sizes[l])
            per_row = src if nnz_per_row is None else min(src, nnz_per_row)
            self.bounds.insert(0, (rows, src, max(1, rows * per_row)))
            rows = src
        self.src_ids, self.indptr, self.indices, self.edge_w = [], [], [], []
        self.sizes = torch.zeros((self.L, 4), dtype=torch.int64, device=device)
        self.c = (CBlock * self.L)()
        for l, (cd, cs, cn) in enumerate(self.bounds):
            self.src_ids.append(torch.empty(max(cs, 1), dtype=graph.idx_dtype, device=device))
            self.indptr.append(torch.empty(cd + 1, dtype=torch.int32, device=device))
            self.indices.append(torch.empty(cn, dtype=torch.int32, device=device))
            self.edge_w.append(torch.empty(cn, dtype=torch.float32, device=device))
            self.c[l] = CBlock(cd, cs, cn, self.src_ids[l].data_ptr(), self.indptr[l].data_ptr(),
                               self.indices[l].data_ptr(), self.sizes[l].data_ptr())
        self.edge_w_ptrs = (_vp * self.L)(*[t.data_ptr() for t in self.edge_w])


class Cache:
    """Feature storage plus the HBM cache of hot rows.  `feats` may be a pinned host tensor
    or a device tensor; with num_cached=None there is no cache and feats is read directly."""

    def __init__(self, graph: Graph, feats: torch.Tensor, num_cached: Optional[int], cache_stride: Optional[int] = None):
        assert feats.dim() == 2 and feats.stride(1) == 1
        assert feats.is_cuda or feats.is_pinned(), "feats must be device or pinned host memory"
        self.feats = feats
        self.dim = feats.shape[1]
        dev = graph.col_idx.device
        self.num_cached = num_cached
        if num_cached is None:
            self.cache_rows = self.slot_of = self.cached_ids = None
            self.cache_stride = 0
            nc = 0
        else:
            nc = int(num_cached)
            self.cache_stride = int(cache_stride or self.dim)
            self.cache_rows = torch.zeros((max(nc, 1), self.cache_stride), dtype=feats.dtype, device=dev)
            self.slot_of = torch.empty(max(graph.num_nodes, 1), dtype=torch.int32, device=dev)
            self.cached_ids = torch.empty(max(nc, 1), dtype=graph.idx_dtype, device=dev)
        self.c = CCache(graph.num_nodes, nc, self.dim, _dtype(feats), feats.data_ptr(), feats.stride(0),
                        _ptr(self.cache_rows), self.cache_stride, _ptr(self.slot_of), _ptr(self.cached_ids))


# ---------------------------------------------------------------------------------- the four calls

def mqg_build_cache(ctx: Context, graph: Graph, cache: Cache, stream=None) -> None:
    ctx.check(lib.mqg_build_cache(ctx.h, ctypes.byref(graph.c), ctypes.byref(cache.c), _stream(stream)))


def mqg_build_cache_ex(ctx: Context, graph: Graph, cache: Cache, policy: int, *, seed: int = 0,
                       train_ids: Optional[torch.Tensor] = None, step_fanouts: Sequence[int] = (),
                       scores_out: Optional[torch.Tensor] = None, walk_form: int = MQG_WALK_PUSH,
                       graph_symmetric: bool = False, stream=None) -> None:
    """Cache filled by one of the policies MQG_CACHE_*."""
    fo = (_i32 * max(1, len(step_fanouts)))(*step_fanouts)
    if train_ids is not None:
        assert train_ids.is_cuda and train_ids.dtype == graph.idx_dtype and train_ids.is_contiguous()
    if scores_out is not None:
        assert scores_out.is_cuda and scores_out.dtype == torch.float64 and scores_out.numel() >= graph.num_nodes
    plan = CCachePlan(policy, len(step_fanouts), seed & 0xFFFFFFFFFFFFFFFF, _ptr(train_ids),
                      0 if train_ids is None else train_ids.numel(), fo, _ptr(scores_out), walk_form,
                      1 if graph_symmetric else 0)
    ctx.check(lib.mqg_build_cache_ex(ctx.h, ctypes.byref(graph.c), ctypes.byref(cache.c), ctypes.byref(plan),
                                     _stream(stream)))


def mqg_sample_blocks(ctx: Context, graph: Graph, seeds: torch.Tensor, fanouts: Sequence[int], rng_seed: int,
                      blocks: Blocks, stream=None) -> None:
    assert seeds.is_cuda and seeds.dtype == graph.idx_dtype and seeds.is_contiguous()
    arr = (_i32 * len(fanouts))(*fanouts)
    ctx.check(lib.mqg_sample_blocks(ctx.h, ctypes.byref(graph.c), seeds.data_ptr(), seeds.numel(), arr,
                                    len(fanouts), ctypes.c_uint64(rng_seed & 0xFFFFFFFFFFFFFFFF), blocks.c,
                                    _stream(stream)))


def mqg_sample_blocks_seed_dev(ctx: Context, graph: Graph, seeds: torch.Tensor, fanouts: Sequence[int],
                               rng_seed_dev: torch.Tensor, blocks: Blocks, stream=None) -> None:
    """As mqg_sample_blocks, the seed read from a one-element device int64 tensor at run time."""
    assert seeds.is_cuda and seeds.dtype == graph.idx_dtype and seeds.is_contiguous()
    assert rng_seed_dev.is_cuda and rng_seed_dev.dtype == torch.int64 and rng_seed_dev.numel() >= 1
    arr = (_i32 * len(fanouts))(*fanouts)
    ctx.check(lib.mqg_sample_blocks_seed_dev(ctx.h, ctypes.byref(graph.c), seeds.data_ptr(), seeds.numel(), arr,
                                             len(fanouts), rng_seed_dev.data_ptr(), blocks.c, _stream(stream)))


def mqg_sample_layerwise(ctx: Context, graph: Graph, seeds: torch.Tensor, layer_sizes: Sequence[int], rng_seed: int,
                         blocks: "LayerwiseBlocks", normalise: bool = True, method: int = 0, stream=None) -> None:
    assert seeds.is_cuda and seeds.dtype == graph.idx_dtype and seeds.is_contiguous()
    arr = (_i32 * len(layer_sizes))(*layer_sizes)
    ctx.check(lib.mqg_sample_layerwise(ctx.h, ctypes.byref(graph.c), seeds.data_ptr() if seeds.numel() else None,
                                       seeds.numel(), arr, len(layer_sizes), rng_seed & 0xFFFFFFFFFFFFFFFF,
                                       1 if normalise else 0, method, blocks.c, blocks.edge_w_ptrs, _stream(stream)))


def mqg_select_smallest_keys(ctx: Context, keys: torch.Tensor, k: int, stream=None) -> torch.Tensor:
    """keys: device int64 tensor holding unsigned 64-bit patterns.  Returns a bool tensor: selected."""
    assert keys.is_cuda and keys.dtype == torch.int64 and keys.is_contiguous()
    n = keys.numel()
    words = torch.empty(max(1, (n + 31) // 32), dtype=torch.int32, device=keys.device)
    ctx.check(lib.mqg_select_smallest_keys(ctx.h, keys.data_ptr() if n else None, n, k, words.data_ptr(), _stream(stream)))
    bits = (words.view(-1, 1) >> torch.arange(32, device=keys.device, dtype=torch.int32)) & 1
    return bits.reshape(-1)[:n].bool()


def mqg_select_row_candidates(ctx: Context, keys: torch.Tensor, slot_words: torch.Tensor, k: int, prioritised: bool = False,
                              ordered: bool = True, stream=None) -> torch.Tensor:
    """keys: device int64 (unsigned 64-bit patterns); slot_words: device int32 (bit 31 = comes after
    every unmarked candidate when prioritised).  Returns a bool tensor: candidate chosen."""
    assert keys.is_cuda and keys.dtype == torch.int64 and keys.is_contiguous()
    assert slot_words.is_cuda and slot_words.dtype == torch.int32 and slot_words.numel() == keys.numel()
    n = keys.numel()
    words = torch.zeros(8, dtype=torch.int32, device=keys.device)
    ctx.check(lib.mqg_select_row_candidates(ctx.h, keys.data_ptr(), slot_words.data_ptr(), n, k, int(prioritised), int(ordered),
                                            words.data_ptr(), _stream(stream)))
    bits = (words.view(-1, 1) >> torch.arange(32, device=keys.device, dtype=torch.int32)) & 1
    return bits.reshape(-1)[:n].bool()


def mqg_exp_tickets(ctx: Context, seed: int, tag: int, first: int, n: int, stream=None) -> torch.Tensor:
    """The race tickets of nodes first .. first + n - 1 in key domain `tag`, as int64 bit patterns."""
    out = torch.empty(max(1, n), dtype=torch.int64, device="cuda")
    ctx.check(lib.mqg_exp_tickets(ctx.h, ctypes.c_uint64(seed & 0xFFFFFFFFFFFFFFFF), tag, first, n, out.data_ptr(),
                                  _stream(stream)))
    return out[:n]


def mqg_gather_features(ctx: Context, cache: Cache, ids: torch.Tensor, num_ids: torch.Tensor, out: torch.Tensor,
                        stats: Optional[torch.Tensor] = None, cap_ids: Optional[int] = None, stream=None) -> None:
    """ids: device id tensor; num_ids: device int64 scalar tensor (e.g. blocks.sizes[0, 1:2])."""
    assert ids.is_cuda and num_ids.is_cuda and num_ids.dtype == torch.int64 and out.is_cuda
    assert out.dtype == cache.feats.dtype and out.stride(1) == 1
    cap = int(cap_ids if cap_ids is not None else min(ids.numel(), out.shape[0]))
    assert cap <= ids.numel() and cap <= out.shape[0]
    ctx.check(lib.mqg_gather_features(ctx.h, ctypes.byref(cache.c), _itype(ids), ids.data_ptr(), num_ids.data_ptr(),
                                      cap, out.data_ptr(), out.stride(0), _ptr(stats), _stream(stream)))


def _gather_half(fn, ctx, cache, ids, num_ids, out, stats, cap_ids, stream):
    assert ids.is_cuda and num_ids.is_cuda and num_ids.dtype == torch.int64 and out.is_cuda
    assert out.dtype == cache.feats.dtype and out.stride(1) == 1
    cap = int(cap_ids if cap_ids is not None else min(ids.numel(), out.shape[0]))
    assert cap <= ids.numel() and cap <= out.shape[0]
    ctx.check(fn(ctx.h, ctypes.byref(cache.c), _itype(ids), ids.data_ptr(), num_ids.data_ptr(), cap, out.data_ptr(),
                 out.stride(0), _ptr(stats), _stream(stream)))


def mqg_gather_features_cached(ctx: Context, cache: Cache, ids: torch.Tensor, num_ids: torch.Tensor, out: torch.Tensor,
                               stats: Optional[torch.Tensor] = None, cap_ids: Optional[int] = None, stream=None) -> None:
    """First half of mqg_gather_features: classify the ids, copy the cached rows."""
    _gather_half(lib.mqg_gather_features_cached, ctx, cache, ids, num_ids, out, stats, cap_ids, stream)


def mqg_gather_features_missed(ctx: Context, cache: Cache, ids: torch.Tensor, num_ids: torch.Tensor, out: torch.Tensor,
                               stats: Optional[torch.Tensor] = None, cap_ids: Optional[int] = None, stream=None) -> None:
    """Second half: copy the rows the first half did not find in the cache."""
    _gather_half(lib.mqg_gather_features_missed, ctx, cache, ids, num_ids, out, stats, cap_ids, stream)


def mqg_gather_features_static(cache: Cache, ids: torch.Tensor, num_ids: torch.Tensor, out: torch.Tensor,
                               stats: Optional[torch.Tensor] = None, cap_ids: Optional[int] = None, stream=None) -> None:
    """mqg_gather_features without a context: the library's fixed device array holds the lists."""
    assert ids.is_cuda and num_ids.is_cuda and num_ids.dtype == torch.int64 and out.is_cuda
    assert out.dtype == cache.feats.dtype and out.stride(1) == 1
    cap = int(cap_ids if cap_ids is not None else min(ids.numel(), out.shape[0]))
    assert cap <= ids.numel() and cap <= out.shape[0]
    rc = lib.mqg_gather_features_static(ctypes.byref(cache.c), _itype(ids), ids.data_ptr(), num_ids.data_ptr(), cap,
                                        out.data_ptr(), out.stride(0), _ptr(stats), _stream(stream))
    if rc != MQG_OK:
        raise MqgError(rc, lib.mqg_last_error(None).decode())


def mqg_sage_mean_aggregate(ctx: Context, blocks: Blocks, l: int, x_src: torch.Tensor, out: torch.Tensor,
                            stream=None) -> None:
    assert x_src.is_cuda and out.is_cuda and x_src.dtype == out.dtype
    assert x_src.stride(1) == 1 and out.stride(1) == 1 and x_src.shape[1] == out.shape[1]
    assert out.shape[0] >= blocks.c[l].cap_dst
    ctx.check(lib.mqg_sage_mean_aggregate(ctx.h, ctypes.byref(blocks.c[l]), x_src.data_ptr(), x_src.stride(0),
                                          out.data_ptr(), out.stride(0), x_src.shape[1], _dtype(x_src),
                                          _stream(stream)))


def mqg_sage_mean_aggregate_backward(ctx: Context, blocks: Blocks, l: int, grad_out: torch.Tensor, grad_x: torch.Tensor,
                                     stream=None) -> None:
    """grad_out: [>= num_dst, dim] gradient of the block's output; grad_x: [>= cap_src, dim] receives the
    gradient with respect to the block's source rows."""
    assert grad_out.is_cuda and grad_x.is_cuda and grad_out.dtype == grad_x.dtype
    assert grad_out.stride(1) == 1 and grad_x.stride(1) == 1 and grad_out.shape[1] == grad_x.shape[1]
    assert grad_x.shape[0] >= blocks.c[l].cap_src
    ctx.check(lib.mqg_sage_mean_aggregate_backward(ctx.h, ctypes.byref(blocks.c[l]), grad_out.data_ptr(),
                                                   grad_out.stride(0), grad_x.data_ptr(), grad_x.stride(0),
                                                   grad_x.shape[1], _dtype(grad_x), _stream(stream)))


def mqg_gcn_edge_weights(ctx: Context, graph: Graph, blocks: Blocks, l: int, edge_w: torch.Tensor, self_w: torch.Tensor,
                         stream=None) -> None:
    """edge_w: [>= cap_nnz] float32, self_w: [>= cap_dst] float32 (device)."""
    for t, cap in ((edge_w, blocks.c[l].cap_nnz), (self_w, blocks.c[l].cap_dst)):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() >= cap
    ctx.check(lib.mqg_gcn_edge_weights(ctx.h, ctypes.byref(graph.c), ctypes.byref(blocks.c[l]), edge_w.data_ptr(),
                                       self_w.data_ptr(), _stream(stream)))


def _weights(edge_w, self_w):
    assert edge_w.is_cuda and edge_w.dtype == torch.float32 and edge_w.is_contiguous()
    if self_w is not None:
        assert self_w.is_cuda and self_w.dtype == torch.float32 and self_w.is_contiguous()
    return edge_w.data_ptr(), (self_w.data_ptr() if self_w is not None else None)


def mqg_weighted_aggregate(ctx: Context, blocks: Blocks, l: int, edge_w: torch.Tensor, self_w: Optional[torch.Tensor],
                           x: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    assert x.is_cuda and out.is_cuda and x.dtype == out.dtype and x.stride(1) == 1 and out.stride(1) == 1
    assert x.shape[1] == out.shape[1] and out.shape[0] >= blocks.c[l].cap_dst
    assert edge_w.numel() >= blocks.c[l].cap_nnz and (self_w is None or self_w.numel() >= blocks.c[l].cap_dst)
    ew, sw = _weights(edge_w, self_w)
    ctx.check(lib.mqg_weighted_aggregate(ctx.h, ctypes.byref(blocks.c[l]), ew, sw, x.data_ptr(), x.stride(0),
                                         out.data_ptr(), out.stride(0), x.shape[1], _dtype(x), _stream(stream)))


def mqg_weighted_aggregate_backward(ctx: Context, blocks: Blocks, l: int, edge_w: torch.Tensor,
                                    self_w: Optional[torch.Tensor], grad_out: torch.Tensor, grad_x: torch.Tensor,
                                    stream=None) -> None:
    assert grad_out.is_cuda and grad_x.is_cuda and grad_out.dtype == grad_x.dtype
    assert grad_out.stride(1) == 1 and grad_x.stride(1) == 1 and grad_out.shape[1] == grad_x.shape[1]
    assert grad_x.shape[0] >= blocks.c[l].cap_src
    assert edge_w.numel() >= blocks.c[l].cap_nnz and (self_w is None or self_w.numel() >= blocks.c[l].cap_dst)
    ew, sw = _weights(edge_w, self_w)
    ctx.check(lib.mqg_weighted_aggregate_backward(ctx.h, ctypes.byref(blocks.c[l]), ew, sw, grad_out.data_ptr(),
                                                  grad_out.stride(0), grad_x.data_ptr(), grad_x.stride(0),
                                                  grad_x.shape[1], _dtype(grad_x), _stream(stream)))


def mqg_queue_size(max_prepare_ms: float, mean_compute_ms: float, total_mem_bytes: int, peak_mem_bytes: int,
                   margin_percent: int, mem_per_batch_bytes: int):
    """Returns (queue_size, cap) of the paper's queue-sizing rule; host arithmetic in the library."""
    cap, q = _i64(0), _i64(0)
    rc = lib.mqg_queue_size(max_prepare_ms, mean_compute_ms, total_mem_bytes, peak_mem_bytes, margin_percent,
                            mem_per_batch_bytes, ctypes.byref(cap), ctypes.byref(q))
    if rc != MQG_OK:
        raise MqgError(rc, lib.mqg_last_error(None).decode())
    return q.value, cap.value
