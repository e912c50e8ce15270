"""ctypes binding of the C ABI in include/legend.h: argument marshalling only.

Every function here has the name of the C entry point it calls.  There is no
CPU fallback: if the shared library is missing the import of this module fails.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LEGEND_HIP_LIB selects another build of the same library (e.g. one compiled with debug flags)
LIB_PATH = os.environ.get("LEGEND_HIP_LIB") or os.path.join(_HERE, "liblegend_hip.so")

LEGEND_OK = 0
LEGEND_E_INVAL, LEGEND_E_NOMEM, LEGEND_E_NOT_RESIDENT = -1, -2, -3
LEGEND_E_RANGE, LEGEND_E_HIP, LEGEND_E_STATE = -4, -5, -6
SCORE_DOT, SCORE_DISTMULT, SCORE_COMPLEX, SCORE_TRANSE_L1 = 0, 1, 2, 3
LOSS_SOFTMAX, LOSS_LOGISTIC, LOSS_SOFTMAX_POS, LOSS_MARGIN = 0, 1, 2, 3
CORRUPT_DST, CORRUPT_SRC, CORRUPT_BOTH = 0, 1, 2
UPDATE_DETERMINISTIC, UPDATE_ATOMIC = 0, 1
MEM_HOST, MEM_DEVICE = 0, 1
TABLE_NODE_EMB, TABLE_NODE_STATE, TABLE_REL_EMB, TABLE_REL_STATE = 0, 1, 2, 3

EXPORTS = [
    "legend_init_partitions", "legend_destroy", "legend_swap_partition", "legend_partition_slot",
    "legend_train_bucket", "legend_train_bucket_range", "legend_train_epoch", "legend_score_edges", "legend_rank_edges", "legend_rank_edges_static",
    "legend_rank_edges_static_max_triples", "legend_read_embeddings", "legend_debug_batch_indices",
    "legend_plan_order", "legend_sync", "legend_profile_enable", "legend_profile_read",
    "legend_profile_name", "legend_batch_shape_of", "legend_unique_rows_read", "legend_fallback_chunks_read",
    "legend_last_error",
]


class legend_config(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("device", C.c_int32), ("num_nodes", C.c_int64),
        ("num_relations", C.c_int32), ("dim", C.c_int32), ("num_partitions", C.c_int32),
        ("buffer_capacity", C.c_int32), ("score", C.c_int32), ("loss", C.c_int32),
        ("corrupt", C.c_int32), ("update_mode", C.c_int32), ("batch_size", C.c_int32),
        ("chunk_size", C.c_int32), ("num_negs", C.c_int32), ("num_degree_negs", C.c_int32),
        ("lr", C.c_float), ("eps", C.c_float), ("neg_weight", C.c_float), ("init_std", C.c_float),
        ("margin", C.c_float), ("seed", C.c_uint64), ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p),
    ]


class legend_prefetch(C.Structure):
    _fields_ = [("evict", C.c_int32), ("load", C.c_int32)]


class legend_rank_metrics(C.Structure):
    _fields_ = [("mrr", C.c_double), ("hits1", C.c_double), ("hits3", C.c_double), ("hits10", C.c_double),
                ("ms", C.c_float)]


class legend_bucket_stats(C.Structure):
    _fields_ = [("loss_sum", C.c_double), ("batches", C.c_int64), ("edges", C.c_int64), ("ms", C.c_double)]


class legend_epoch_stats(C.Structure):
    _fields_ = [("loss_sum", C.c_double), ("edges", C.c_int64), ("batches", C.c_int64), ("swaps", C.c_int64),
                ("buffer_states", C.c_int64), ("bytes_per_swap", C.c_int64), ("ms", C.c_double)]


class legend_batch_shape(C.Structure):
    _fields_ = [("occurrences", C.c_int64), ("neg_rows", C.c_int64), ("workspace_bytes", C.c_int64),
                ("key_bits", C.c_int32), ("row_tiles", C.c_int32)]


class LegendError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"legend error {code}: {message}")
        self.code = code


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2505_09258_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.legend_init_partitions.argtypes = [C.POINTER(legend_config), vp, vp, C.POINTER(vp)]
    lib.legend_destroy.argtypes = [vp]
    lib.legend_swap_partition.argtypes = [vp, i32, i32]
    lib.legend_partition_slot.argtypes = [vp, i32, C.POINTER(i32)]
    lib.legend_train_bucket.argtypes = [vp, i32, i32, vp, i64, i32, i32, C.POINTER(legend_prefetch),
                                        C.POINTER(legend_bucket_stats)]
    lib.legend_train_bucket_range.argtypes = [vp, i32, i32, vp, i64, i32, i32, i64, i64, C.POINTER(legend_prefetch),
                                              C.POINTER(legend_bucket_stats)]
    lib.legend_train_epoch.argtypes = [vp, vp, vp, i32, i32, i32, C.POINTER(legend_epoch_stats)]
    lib.legend_score_edges.argtypes = [vp, vp, vp, vp, i64, vp]
    lib.legend_rank_edges.argtypes = [vp, vp, vp, vp, i64, i32, vp, i64, vp, vp, C.POINTER(legend_rank_metrics)]
    lib.legend_rank_edges_static.argtypes = [vp, vp, vp, vp, i64, i32, vp, i64, vp, vp, vp, vp]
    lib.legend_rank_edges_static_max_triples.argtypes = [i32]
    lib.legend_read_embeddings.argtypes = [vp, i32, vp, i64, vp]
    lib.legend_debug_batch_indices.argtypes = [vp, i32, i32, vp, i64, i32, i32, i64, vp, i64, vp, i64,
                                               C.POINTER(i64)]
    lib.legend_plan_order.argtypes = [i32, vp, i32, C.POINTER(i32), vp, vp, vp]
    lib.legend_sync.argtypes = [vp]
    lib.legend_profile_enable.argtypes = [vp, C.c_uint32]
    lib.legend_profile_read.argtypes = [vp, vp, vp, i32]
    lib.legend_profile_name.argtypes = [i32]
    lib.legend_profile_name.restype = C.c_char_p
    lib.legend_batch_shape_of.argtypes = [vp, C.POINTER(legend_batch_shape)]
    lib.legend_unique_rows_read.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
    lib.legend_fallback_chunks_read.argtypes = [vp, C.POINTER(i64)]
    lib.legend_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("legend_profile_name", "legend_last_error", "legend_rank_edges_static_max_triples"):
            getattr(lib, name).restype = C.c_int
    lib.legend_rank_edges_static_max_triples.restype = C.c_int64
    return lib


_lib = _load()


def legend_last_error() -> str:
    return _lib.legend_last_error().decode()


def _check(rc: int) -> None:
    if rc != LEGEND_OK:
        raise LegendError(rc, legend_last_error())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _as(a, dtype) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def make_config(*, num_nodes, dim, num_partitions=1, buffer_capacity=None, num_relations=0, score=SCORE_DOT,
                loss=LOSS_SOFTMAX, corrupt=CORRUPT_DST, update_mode=UPDATE_DETERMINISTIC, batch_size, chunk_size,
                num_negs, num_degree_negs=0, lr=0.1, eps=1e-10, neg_weight=-1.0, init_std=1e-3, margin=1.0, seed=0, device=0,
                compute_stream=None, copy_stream=None) -> legend_config:
    cfg = legend_config()
    cfg.struct_size = C.sizeof(legend_config)
    cfg.device = device
    cfg.num_nodes = num_nodes
    cfg.num_relations = num_relations
    cfg.dim = dim
    cfg.num_partitions = num_partitions
    cfg.buffer_capacity = num_partitions if buffer_capacity is None else buffer_capacity
    cfg.score, cfg.loss, cfg.corrupt, cfg.update_mode = score, loss, corrupt, update_mode
    cfg.batch_size, cfg.chunk_size, cfg.num_negs, cfg.num_degree_negs = batch_size, chunk_size, num_negs, num_degree_negs
    cfg.lr, cfg.eps, cfg.neg_weight, cfg.init_std, cfg.margin = lr, eps, neg_weight, init_std, margin
    cfg.seed = seed & ((1 << 64) - 1)
    cfg.compute_stream = compute_stream
    cfg.copy_stream = copy_stream
    return cfg


def legend_init_partitions(cfg: legend_config, init_node_emb: np.ndarray, init_rel_emb: Optional[np.ndarray]):
    node = _as(init_node_emb, np.float32)
    rel = _as(init_rel_emb, np.float32)
    if node is not None and node.shape != (cfg.num_nodes, cfg.dim):
        raise ValueError("init_node_emb must be [num_nodes, dim]")
    if rel is not None and rel.shape != (max(cfg.num_relations, 1), cfg.dim):
        raise ValueError("init_rel_emb must be [max(num_relations,1), dim]")
    handle = C.c_void_p()
    _check(_lib.legend_init_partitions(C.byref(cfg), _ptr(node), _ptr(rel), C.byref(handle)))
    return handle


def legend_destroy(ctx) -> None:
    _check(_lib.legend_destroy(ctx))


def legend_swap_partition(ctx, evict: int, load: int) -> None:
    _check(_lib.legend_swap_partition(ctx, evict, load))


def legend_partition_slot(ctx, part: int) -> int:
    out = C.c_int32(-2)
    _check(_lib.legend_partition_slot(ctx, part, C.byref(out)))
    return out.value


def legend_train_bucket(ctx, src_part: int, dst_part: int, edges, m: Optional[int] = None, edges_mem: int = MEM_HOST,
                        epoch: int = 0, hint: Optional[Sequence[int]] = None, want_stats: bool = True):
    """edges: int32 [m,3] numpy array (host) or an integer device address with m given."""
    return legend_train_bucket_range(ctx, src_part, dst_part, edges, m, edges_mem, epoch, 0, -1, hint, want_stats,
                                     _whole=True)


def legend_train_bucket_range(ctx, src_part: int, dst_part: int, edges, m: Optional[int] = None,
                              edges_mem: int = MEM_HOST, epoch: int = 0, batch_begin: int = 0, batch_end: int = -1,
                              hint: Optional[Sequence[int]] = None, want_stats: bool = True, _whole: bool = False):
    if edges_mem == MEM_HOST:
        e = _as(edges, np.int32)
        if e.ndim != 2 or e.shape[1] != 3:
            raise ValueError("edges must be [m, 3]")
        m = e.shape[0]
        eptr = _ptr(e)
    else:
        eptr = C.c_void_p(int(edges))
    h = None
    if hint is not None:
        h = legend_prefetch(int(hint[0]), int(hint[1]))
    st = legend_bucket_stats() if want_stats else None
    hp = C.byref(h) if h is not None else None
    sp = C.byref(st) if st is not None else None
    if _whole:
        _check(_lib.legend_train_bucket(ctx, src_part, dst_part, eptr, m, edges_mem, epoch, hp, sp))
    else:
        _check(_lib.legend_train_bucket_range(ctx, src_part, dst_part, eptr, m, edges_mem, epoch, batch_begin,
                                              batch_end, hp, sp))
    if st is None:
        return None
    return dict(loss_sum=st.loss_sum, batches=st.batches, edges=st.edges, ms=st.ms)


def legend_train_epoch(ctx, n: int, buckets, edges_mem: int = MEM_HOST, epoch: int = 0, overlap: bool = True):
    """buckets: {(i, j): int32 [m,3] array} for MEM_HOST, or {(i, j): (device address, m)} for MEM_DEVICE."""
    ptrs = (C.c_void_p * (n * n))()
    sizes = (C.c_int64 * (n * n))()
    keep = []
    for (i, j), e in buckets.items():
        if edges_mem == MEM_HOST:
            a = _as(e, np.int32)
            keep.append(a)
            ptrs[i * n + j] = a.ctypes.data if a.shape[0] else None
            sizes[i * n + j] = a.shape[0]
        else:
            ptrs[i * n + j] = int(e[0]) if e[1] else None
            sizes[i * n + j] = int(e[1])
    st = legend_epoch_stats()
    _check(_lib.legend_train_epoch(ctx, ptrs, sizes, edges_mem, epoch, 1 if overlap else 0, C.byref(st)))
    return {k: getattr(st, k) for k, _ in legend_epoch_stats._fields_}


def legend_score_edges(ctx, src, rel, dst) -> np.ndarray:
    s = _as(src, np.int64)
    d = _as(dst, np.int64)
    r = _as(rel, np.int32)
    out = np.empty(s.shape[0], np.float32)
    _check(_lib.legend_score_edges(ctx, _ptr(s), _ptr(r), _ptr(d), s.shape[0], _ptr(out)))
    return out


def legend_rank_edges(ctx, src, rel, dst, side: int = CORRUPT_DST, candidates=None):
    """(greater, equal, metrics) of the triples against the candidates (None: all nodes)."""
    s = _as(src, np.int64)
    d = _as(dst, np.int64)
    r = _as(rel, np.int32)
    cand = _as(candidates, np.int64)
    if cand is not None and cand.shape[0] == 0:
        cand = np.zeros(1, np.int64)[:0]          # an empty list still needs a non-NULL pointer (NULL means all nodes)
    m = s.shape[0]
    greater = np.empty(m, np.int32)
    equal = np.empty(m, np.int32)
    mt = legend_rank_metrics()
    _check(_lib.legend_rank_edges(ctx, _ptr(s), _ptr(r), _ptr(d), m, side, _ptr(cand),
                                  0 if cand is None else cand.shape[0], _ptr(greater), _ptr(equal), C.byref(mt)))
    return greater, equal, {k: getattr(mt, k) for k, _ in legend_rank_metrics._fields_}


def legend_rank_edges_static(ctx, src: int, rel: Optional[int], dst: int, m: int, side: int, candidates: Optional[int],
                             num_candidates: int, greater: int, equal: int, metrics: int, status: int) -> None:
    """Every array argument is a device address (an integer); None for rel / candidates passes NULL."""
    def dp(a):
        return None if a is None else C.c_void_p(int(a))
    _check(_lib.legend_rank_edges_static(ctx, dp(src), dp(rel), dp(dst), m, side, dp(candidates), num_candidates,
                                         dp(greater), dp(equal), dp(metrics), dp(status)))


def legend_rank_edges_static_max_triples(dim: int) -> int:
    return int(_lib.legend_rank_edges_static_max_triples(dim))


def legend_read_embeddings(ctx, table: int, ids, m: int, dim: int) -> np.ndarray:
    i = _as(ids, np.int64)
    if i is not None:
        m = i.shape[0]
    out = np.empty((m, dim), np.float32)
    _check(_lib.legend_read_embeddings(ctx, table, _ptr(i), m, _ptr(out)))
    return out


def legend_debug_batch_indices(ctx, src_part, dst_part, edges, epoch, batch, neg_capacity, touched_capacity,
                               m: Optional[int] = None, edges_mem: int = MEM_HOST):
    if edges_mem == MEM_HOST:
        e = _as(edges, np.int32)
        m = e.shape[0]
        eptr = _ptr(e)
    else:
        eptr = C.c_void_p(int(edges))
    neg = np.empty(neg_capacity, np.int32)
    touched = np.empty(touched_capacity, np.int64)
    cnt = C.c_int64(0)
    _check(_lib.legend_debug_batch_indices(ctx, src_part, dst_part, eptr, m, edges_mem, epoch, batch, _ptr(neg),
                                           neg_capacity, _ptr(touched), touched_capacity, C.byref(cnt)))
    return neg, touched[: cnt.value]


def legend_plan_order(n: int):
    cap = max(8, 8 * n * n)
    states = np.empty((cap, 3), np.int32)
    buckets = np.empty((n * n, 2), np.int32)
    begin = np.empty(cap + 1, np.int32)
    overlap = np.empty(cap, np.int32)
    ns = C.c_int32(0)
    rc = _lib.legend_plan_order(n, _ptr(states), cap, C.byref(ns), _ptr(buckets), _ptr(begin), _ptr(overlap))
    if rc != LEGEND_OK:
        raise LegendError(rc, "legend_plan_order failed")
    k = ns.value
    return states[:k].copy(), buckets, begin[: k + 1].copy(), overlap[:k].copy()


def legend_sync(ctx) -> None:
    _check(_lib.legend_sync(ctx))


def legend_profile_enable(ctx, mask: int) -> None:
    _check(_lib.legend_profile_enable(ctx, mask))


def legend_profile_name(k: int) -> Optional[str]:
    s = _lib.legend_profile_name(k)
    return None if s is None else s.decode()


def legend_profile_read(ctx):
    names = []
    k = 0
    while legend_profile_name(k) is not None:
        names.append(legend_profile_name(k))
        k += 1
    ms = np.zeros(k, np.float64)
    launches = np.zeros(k, np.int64)
    _check(_lib.legend_profile_read(ctx, _ptr(ms), _ptr(launches), k))
    return {n: dict(ms=float(ms[i]), launches=int(launches[i])) for i, n in enumerate(names)}


def legend_batch_shape_of(ctx):
    s = legend_batch_shape()
    _check(_lib.legend_batch_shape_of(ctx, C.byref(s)))
    return dict(occurrences=s.occurrences, neg_rows=s.neg_rows, workspace_bytes=s.workspace_bytes,
                key_bits=s.key_bits, row_tiles=s.row_tiles)


def legend_fallback_chunks_read(ctx) -> int:
    n = C.c_int64(0)
    _check(_lib.legend_fallback_chunks_read(ctx, C.byref(n)))
    return int(n.value)


def legend_unique_rows_read(ctx):
    u, b = C.c_int64(0), C.c_int64(0)
    _check(_lib.legend_unique_rows_read(ctx, C.byref(u), C.byref(b)))
    return u.value, b.value
