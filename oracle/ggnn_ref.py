"""ctypes front end of the C oracle (oracle/ggnn_ref.c).  Test infrastructure only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build_oracle

L2, COSINE = 0, 1
F32, U8 = 0, 1
ROW_LANES = 8        # accumulators of the fixed float32 summation tree (see ggnn_ref.c) ...
WIDE_ROW_LANES = 64  # ... and for rows longer than 1024 bytes


def row_lanes(D, itemsize, metric=0):
    """Accumulators of the summation tree for rows of D elements: 8 for rows of at most 1024 bytes
    (cosine: of the float32 unit-length copy), 64 beyond."""
    row_bytes = D * (4 if metric == 1 else itemsize)
    return ROW_LANES if row_bytes <= 1024 else WIDE_ROW_LANES

_lib = None


class BuildParams(C.Structure):
    _fields_ = [("tau_build", C.c_float), ("refinements", C.c_int), ("pq_cap", C.c_int),
                ("visited_cap", C.c_int), ("max_iter", C.c_int), ("sym_constraint", C.c_int)]


def default_params(tau_build=0.5, refinements=2, pq_cap=64, visited_cap=384, max_iter=384, sym_constraint=1):
    return BuildParams(tau_build, refinements, pq_cap, visited_cap, max_iter, sym_constraint)


def lib():
    global _lib
    if _lib is None:
        # GGNN_REF_LIB: an alternative build of the oracle (used by the mutation checks of the pins)
        path = os.environ.get("GGNN_REF_LIB") or build_oracle.build(force=False)
        L = C.CDLL(path)
        vp, i64, i32, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_float
        L.ggnn_ref_geometry.argtypes = [i64, C.c_int, C.c_int, vp, vp, vp]
        L.ggnn_ref_perm.argtypes = [C.c_uint64, i64, i64]
        L.ggnn_ref_perm.restype = i64
        L.ggnn_ref_perm_inv.argtypes = [C.c_uint64, i64, i64]
        L.ggnn_ref_perm_inv.restype = i64
        L.ggnn_ref_uniform.argtypes = [C.c_uint64, C.c_int, i64]
        L.ggnn_ref_uniform.restype = C.c_double
        L.ggnn_ref_distance.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, C.c_int]
        L.ggnn_ref_distance.restype = f32
        L.ggnn_ref_bruteforce.argtypes = [vp, i64, C.c_int, C.c_int, C.c_int, C.c_int, vp, i64, C.c_int, vp, vp]
        L.ggnn_ref_graph_create.argtypes = [vp, i64, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_uint64, C.c_int]
        L.ggnn_ref_graph_create.restype = vp
        L.ggnn_ref_graph_free.argtypes = [vp]
        L.ggnn_ref_graph_free.restype = None
        L.ggnn_ref_graph_g.argtypes = [vp]
        L.ggnn_ref_graph_n.argtypes = [vp, C.c_int]
        L.ggnn_ref_graph_n.restype = i64
        for name in ("edges", "to_lower", "to_base", "inv_count"):
            f = getattr(L, "ggnn_ref_graph_" + name)
            f.argtypes = [vp, C.c_int]
            f.restype = C.POINTER(i32)
        L.ggnn_ref_graph_dnn1.argtypes = [vp]
        L.ggnn_ref_graph_dnn1.restype = C.POINTER(f32)
        L.ggnn_ref_graph_stats.argtypes = [vp]
        L.ggnn_ref_graph_stats.restype = C.POINTER(f32)
        L.ggnn_ref_graph_normalised.argtypes = [vp]
        L.ggnn_ref_graph_normalised.restype = C.POINTER(f32)
        L.ggnn_ref_select.argtypes = [vp, C.c_int]
        L.ggnn_ref_merge.argtypes = [vp, C.c_int, C.c_int, C.POINTER(BuildParams)]
        L.ggnn_ref_sym.argtypes = [vp, C.c_int, C.POINTER(BuildParams)]
        L.ggnn_ref_build.argtypes = [vp, C.POINTER(BuildParams)]
        L.ggnn_ref_query.argtypes = [vp, vp, i64, C.c_int, C.c_int, f32, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp]
        L.ggnn_ref_num_threads.restype = C.c_int
        L.ggnn_ref_set_num_threads.argtypes = [C.c_int]
        L.ggnn_ref_set_num_threads.restype = None
        L.ggnn_ref_query_from.argtypes = [vp, vp, i64, C.c_int, C.c_int, f32, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_int, vp, vp, vp]
        L.ggnn_ref_merge_shards.argtypes = [C.c_int, i64, C.c_int, vp, vp, vp, vp, vp]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _dtype_code(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint8:
        return U8
    raise TypeError(a.dtype)


def geometry(N, s, L):
    g = np.zeros(1, np.int32)
    n = np.zeros(L, np.int64)
    G = np.zeros(L, np.int64)
    rc = lib().ggnn_ref_geometry(N, s, L, _ptr(g), _ptr(n), _ptr(G))
    if rc != 0:
        raise ValueError("no valid hierarchy for N=%d s=%d L=%d" % (N, s, L))
    return int(g[0]), n.tolist(), G.tolist()


def perm(seed, N, p):
    return lib().ggnn_ref_perm(seed, N, p)


def perm_inv(seed, N, row):
    return lib().ggnn_ref_perm_inv(seed, N, row)


def uniform(seed, l_top, row):
    return lib().ggnn_ref_uniform(seed, l_top, row)


def distance(q, row, metric=L2, lanes=None):
    q = np.ascontiguousarray(q, np.float32)
    row = np.ascontiguousarray(row)
    lanes = lanes or row_lanes(q.shape[0], row.dtype.itemsize, metric)
    return float(lib().ggnn_ref_distance(_ptr(q), _ptr(row), q.shape[0], _dtype_code(row), metric, lanes))


def bruteforce(base, queries, k, metric=L2, lanes=None):
    base = np.ascontiguousarray(base)
    queries = np.ascontiguousarray(queries)
    lanes = lanes or row_lanes(base.shape[1], base.dtype.itemsize, metric)
    assert base.dtype == queries.dtype and base.shape[1] == queries.shape[1]
    Q = queries.shape[0]
    ids = np.empty((Q, k), np.int32)
    dists = np.empty((Q, k), np.float32)
    rc = lib().ggnn_ref_bruteforce(_ptr(base), base.shape[0], base.shape[1], _dtype_code(base), metric, lanes,
                                   _ptr(queries), Q, k, _ptr(ids), _ptr(dists))
    if rc != 0:
        raise RuntimeError("bruteforce failed: %d" % rc)
    return ids, dists


class Graph:
    """Hierarchical kNN graph held by the oracle.  The arrays returned by the accessors
    are views into the oracle's memory (writable: tests use that to load a state)."""

    def __init__(self, base, K, levels, s=32, metric=L2, seed=42, lanes=None):
        self.base = np.ascontiguousarray(base)
        self.N, self.D = self.base.shape
        lanes = lanes or row_lanes(self.D, self.base.dtype.itemsize, metric)
        self.K, self.L, self.s, self.metric, self.seed, self.lanes = K, levels, s, metric, seed, lanes
        self.h = lib().ggnn_ref_graph_create(_ptr(self.base), self.N, self.D, K, levels, s,
                                             _dtype_code(self.base), metric, seed, lanes)
        if not self.h:
            raise ValueError("invalid graph parameters")
        self.g = lib().ggnn_ref_graph_g(self.h)
        self.n = [lib().ggnn_ref_graph_n(self.h, l) for l in range(levels)]

    def __del__(self):
        try:
            if getattr(self, "h", None) and _lib is not None:
                _lib.ggnn_ref_graph_free(self.h)
                self.h = None
        except Exception:  # interpreter shutdown
            pass

    def _arr(self, fn, layer, shape):
        p = fn(self.h, layer)
        return np.ctypeslib.as_array(p, shape=shape)

    def edges(self, layer):
        return self._arr(lib().ggnn_ref_graph_edges, layer, (self.n[layer], self.K))

    def to_lower(self, layer):
        return self._arr(lib().ggnn_ref_graph_to_lower, layer, (self.n[layer],))

    def to_base(self, layer):
        return self._arr(lib().ggnn_ref_graph_to_base, layer, (self.n[layer],))

    def inv_count(self, layer):
        return self._arr(lib().ggnn_ref_graph_inv_count, layer, (self.n[layer],))

    def dnn1(self):
        return np.ctypeslib.as_array(lib().ggnn_ref_graph_dnn1(self.h), shape=(self.N,))

    def stats(self):
        return np.ctypeslib.as_array(lib().ggnn_ref_graph_stats(self.h), shape=(2,))

    def normalised(self):
        p = lib().ggnn_ref_graph_normalised(self.h)
        return np.ctypeslib.as_array(p, shape=(self.N, self.D)) if p else None

    def select(self, l_top):
        rc = lib().ggnn_ref_select(self.h, l_top)
        assert rc == 0, rc

    def merge(self, l_top, l_m, params):
        rc = lib().ggnn_ref_merge(self.h, l_top, l_m, C.byref(params))
        assert rc == 0, rc

    def sym(self, layer, params):
        rc = lib().ggnn_ref_sym(self.h, layer, C.byref(params))
        assert rc == 0, rc

    def build(self, params=None):
        params = params or default_params()
        rc = lib().ggnn_ref_build(self.h, C.byref(params))
        assert rc == 0, rc
        return self

    def query(self, queries, k, beam, slack, pq_cap=64, visited_cap=384, max_iter=None, every_layer=False,
              counters=False, start_ids=None):
        queries = np.ascontiguousarray(queries)
        assert queries.dtype == self.base.dtype
        Q = queries.shape[0]
        B = max(beam, k)
        max_iter = visited_cap if max_iter is None else max_iter
        ids = np.empty((Q, k), np.int32)
        dists = np.empty((Q, k), np.float32)
        cnt = np.zeros((Q, 2), np.uint32) if counters else None
        st = None if start_ids is None else np.ascontiguousarray(start_ids, np.int32)
        rc = lib().ggnn_ref_query_from(self.h, _ptr(queries), Q, k, B, slack, pq_cap, visited_cap, max_iter,
                                  1 if every_layer else 0, None if st is None else _ptr(st), 0 if st is None else len(st),
                                  _ptr(ids), _ptr(dists), _ptr(cnt) if counters else None)
        if rc != 0:
            raise RuntimeError("query failed: %d" % rc)
        return (ids, dists, cnt) if counters else (ids, dists)


def merge_shards(ids, dists, offsets):
    """ids, dists: S x Q x k per-shard answers; offsets: S shard offsets.  Returns the merged Q x k."""
    ids = np.ascontiguousarray(ids, np.int32)
    dists = np.ascontiguousarray(dists, np.float32)
    offsets = np.ascontiguousarray(offsets, np.int32)
    S, Q, k = ids.shape
    out_i = np.empty((Q, k), np.int32)
    out_d = np.empty((Q, k), np.float32)
    rc = lib().ggnn_ref_merge_shards(S, Q, k, _ptr(ids), _ptr(dists), _ptr(offsets), _ptr(out_i), _ptr(out_d))
    assert rc == 0, rc
    return out_i, out_d


def recall(ids, gt):
    """C@k of the paper's evaluation section: mean overlap of the k returned ids with the k true ones."""
    k = gt.shape[1]
    hit = 0
    for a, b in zip(ids, gt):
        hit += len(set(a[:k].tolist()) & set(b.tolist()))
    return hit / (gt.shape[0] * k)
