"""ctypes binding of libggnn.so (include/ggnn.h): argument marshalling only.

Every function takes torch tensors that live on the GPU (or numpy arrays for the host-side
import / export calls) and passes their addresses on; all computation happens in the library.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

L2, COSINE = 0, 1
F32, U8 = 0, 1
MAX_LEVELS = 8

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libggnn.so")
_lib = None


class GgnnError(RuntimeError):
    pass


class BuildParams(C.Structure):
    _fields_ = [("metric", C.c_int32), ("dtype", C.c_int32), ("segment_size", C.c_int32),
                ("tau_build", C.c_float), ("refinements", C.c_int32), ("pq_cap", C.c_int32),
                ("visited_cap", C.c_int32), ("max_iter", C.c_int32), ("no_sym_constraint", C.c_int32),
                ("stream", C.c_void_p)]


class GraphDesc(C.Structure):
    _fields_ = [("N", C.c_int64), ("D", C.c_int32), ("K", C.c_int32), ("L", C.c_int32), ("s", C.c_int32),
                ("g", C.c_int32), ("dtype", C.c_int32), ("metric", C.c_int32), ("n", C.c_int64 * MAX_LEVELS),
                ("dnn_mean", C.c_float), ("dnn_max", C.c_float), ("graph_bytes", C.c_int64), ("seed", C.c_uint64)]


class QueryParams(C.Structure):
    _fields_ = [("pq_cap", C.c_int32), ("visited_cap", C.c_int32), ("max_iter", C.c_int32), ("every_layer", C.c_int32),
                ("cache_mode", C.c_int32), ("global_visited_min_iter", C.c_int32), ("split_min_queries", C.c_int64),
                ("start_ids_dev", C.c_void_p), ("n_start", C.c_int32), ("asynchronous", C.c_int32), ("stream", C.c_void_p)]


class BuildTimes(C.Structure):
    _fields_ = [("merge_ms", C.c_float), ("sym_ms", C.c_float), ("select_ms", C.c_float),
                ("stats_ms", C.c_float), ("total_ms", C.c_float), ("merge_pops", C.c_uint64),
                ("merge_rows", C.c_uint64), ("sym_pops", C.c_uint64), ("sym_rows", C.c_uint64)]


ProgressFn = C.CFUNCTYPE(None, C.c_char_p, C.c_int32, C.c_int32, C.c_double, C.c_void_p)

EXPORTS = [
    "ggnn_build", "ggnn_build_ex", "ggnn_graph_create", "ggnn_select", "ggnn_merge", "ggnn_sym",
    "ggnn_build_steps", "ggnn_build_set_progress", "ggnn_build_get_times", "ggnn_query", "ggnn_query_ex", "ggnn_query_with", "ggnn_query_static", "ggnn_query_from", "ggnn_graph_info",
    "ggnn_graph_export", "ggnn_graph_import", "ggnn_graph_export_dnn", "ggnn_graph_import_dnn",
    "ggnn_graph_export_inv_count", "ggnn_set_cache_mode", "ggnn_set_split_threshold", "ggnn_set_global_visited_threshold", "ggnn_gather_probe", "ggnn_merge_shards", "ggnn_free", "ggnn_last_error",
]


def lib():
    """Loads libggnn.so.  There is no fallback: without the built library nothing runs."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise GgnnError("%s is missing: run `python -m paper_1912_01059_amd.hipbuild` (or __graft_entry__.build())"
                            % _LIB_PATH)
        L = C.CDLL(_LIB_PATH)
        vp, i64, i32, u64, f32 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64, C.c_float
        L.ggnn_build.argtypes = [vp, i64, i32, i32, i32, u64, C.POINTER(vp)]
        L.ggnn_build_ex.argtypes = [vp, i64, i32, i32, i32, u64, C.POINTER(BuildParams), C.POINTER(vp)]
        L.ggnn_graph_create.argtypes = [vp, i64, i32, i32, i32, u64, C.POINTER(BuildParams), C.POINTER(vp)]
        L.ggnn_select.argtypes = [vp, i32]
        L.ggnn_merge.argtypes = [vp, i32, i32]
        L.ggnn_sym.argtypes = [vp, i32]
        L.ggnn_build_steps.argtypes = [vp]
        L.ggnn_build_set_progress.argtypes = [vp, ProgressFn, vp]
        L.ggnn_build_get_times.argtypes = [vp, C.POINTER(BuildTimes)]
        L.ggnn_query.argtypes = [vp, vp, i64, i32, i32, f32, vp, vp]
        L.ggnn_query_ex.argtypes = [vp, vp, i64, i32, i32, f32, i32, i32, i32, i32, vp, vp, vp, vp, i32]
        L.ggnn_query_with.argtypes = [vp, vp, i64, i32, i32, f32, C.POINTER(QueryParams), vp, vp, vp]
        L.ggnn_query_static.argtypes = [vp, vp, i64, i32, i32, f32, i32, i32, i32, vp, vp, vp, vp, i32]
        L.ggnn_query_from.argtypes = [vp, vp, i64, i32, i32, f32, i32, i32, i32, vp, i32, vp, vp, vp, vp, i32]
        L.ggnn_graph_info.argtypes = [vp, C.POINTER(GraphDesc)]
        L.ggnn_graph_export.argtypes = [vp, i32, vp, vp, vp]
        L.ggnn_graph_import.argtypes = [vp, i32, vp, vp, vp]
        L.ggnn_graph_export_dnn.argtypes = [vp, vp, C.POINTER(f32), C.POINTER(f32)]
        L.ggnn_graph_import_dnn.argtypes = [vp, vp, f32, f32]
        L.ggnn_graph_export_inv_count.argtypes = [vp, i32, vp]
        L.ggnn_set_cache_mode.argtypes = [i32]
        L.ggnn_set_split_threshold.argtypes = [i64]
        L.ggnn_set_global_visited_threshold.argtypes = [C.c_int32]
        L.ggnn_gather_probe.argtypes = [vp, i64, i32, vp, i64, i32, vp, vp]
        L.ggnn_merge_shards.argtypes = [i32, i64, i32, vp, vp, vp, vp, vp, vp, i32]
        L.ggnn_free.argtypes = [vp]
        L.ggnn_free.restype = None
        L.ggnn_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def set_cache_mode(mode: int) -> None:
    """0: best / prioq in registers when they fit (default); 1: always in LDS."""
    _check(lib().ggnn_set_cache_mode(mode))


def set_global_visited_threshold(min_iter: int) -> None:
    """ggnn_set_global_visited_threshold: iteration limit from which user queries keep visited in global memory."""
    _check(lib().ggnn_set_global_visited_threshold(min_iter))


def set_split_threshold(min_queries: int) -> None:
    """Batches of at least this many every-layer queries take the two-launch path (0: default)."""
    _check(lib().ggnn_set_split_threshold(min_queries))


def gather_probe(rows, ids, rows_per_wave, out=None):
    """ggnn_gather_probe on torch's current stream (asynchronous); returns the output tensor."""
    import torch
    n = ids.shape[0]
    waves = (n + rows_per_wave - 1) // rows_per_wave
    if out is None:
        out = torch.empty(waves * 64, dtype=torch.int32, device=rows.device)
    _check(lib().ggnn_gather_probe(_dev_ptr(rows), rows.shape[0], rows.shape[1] * rows.element_size(), _dev_ptr(ids), n,
                                   rows_per_wave, _dev_ptr(out), C.c_void_p(torch.cuda.current_stream().cuda_stream)))
    return out


def merge_shards(ids, dists, offsets):
    """ggnn_merge_shards: ids / dists are S x Q x k GPU tensors, offsets an S int32 GPU tensor."""
    import torch
    S, Q, k = ids.shape
    out_i = torch.empty((Q, k), dtype=torch.int32, device=ids.device)
    out_d = torch.empty((Q, k), dtype=torch.float32, device=ids.device)
    _check(lib().ggnn_merge_shards(S, Q, k, _dev_ptr(ids), _dev_ptr(dists), _dev_ptr(offsets), _dev_ptr(out_i), _dev_ptr(out_d),
                                   C.c_void_p(torch.cuda.current_stream().cuda_stream), 0))
    return out_i, out_d


class ShardedIndex:
    """Sec. 4.5 on one GPU: the base set is cut into S contiguous shards, each with its own graph;
    a query batch is answered on every shard and the answers are merged on the GPU.  The S searches
    are independent: each runs on a stream of its own (default priority), so that the tail of one
    overlaps the start of the next; the merge waits for all of them on the caller's stream."""

    def __init__(self, base, shards, K, levels, progress=None, **build_args):
        import torch
        N = base.shape[0]
        bounds = [N * i // shards for i in range(shards + 1)]
        self.parts = [base[bounds[i]:bounds[i + 1]].contiguous() for i in range(shards)]
        self.offsets = torch.tensor(bounds[:-1], dtype=torch.int32, device=base.device)
        self.graphs = []
        for i, p in enumerate(self.parts):
            self.graphs.append(build(p, K, levels, **build_args))
            if progress is not None:
                progress(i, self.graphs[-1])  # called after each shard's construction
        self.streams = [torch.cuda.Stream(device=base.device) for _ in self.graphs]

    def query(self, queries, k, beam, slack, **query_args):
        import torch
        Q = queries.shape[0]
        S = len(self.graphs)
        ids = torch.empty((S, Q, k), dtype=torch.int32, device=queries.device)
        dists = torch.empty((S, Q, k), dtype=torch.float32, device=queries.device)
        cur = torch.cuda.current_stream(queries.device)
        ready = torch.cuda.Event()
        ready.record(cur)
        for s, g in enumerate(self.graphs):
            st = self.streams[s]
            st.wait_event(ready)
            for t in (queries, ids, dists):
                t.record_stream(st)
            g.query(queries, k, beam, slack, out=(ids[s], dists[s]), stream=st.cuda_stream, asynchronous=True, **query_args)
            done = torch.cuda.Event()
            done.record(st)
            cur.wait_event(done)
        return merge_shards(ids, dists, self.offsets)


def last_error() -> str:
    return lib().ggnn_last_error().decode()


def _check(rc):
    if rc != 0:
        raise GgnnError("ggnn error %d: %s" % (rc, last_error()))


def _dev_ptr(t):
    import torch
    assert isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous(), "need a contiguous GPU tensor"
    return C.c_void_p(t.data_ptr())


def _host_ptr(a):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.c_void_p)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.uint8:
        return U8
    raise TypeError("base must be float32 or uint8, got %s" % t.dtype)


def _params(base, metric, segment_size, tau_build, refinements, pq_cap, visited_cap, max_iter, sym_constraint, stream):
    p = BuildParams()
    p.metric, p.dtype, p.segment_size = metric, _dtype_code(base), segment_size
    p.tau_build = tau_build
    p.refinements = -1 if refinements == 0 else refinements
    p.pq_cap, p.visited_cap, p.max_iter = pq_cap, visited_cap, max_iter
    p.no_sym_constraint = 0 if sym_constraint else 1
    p.stream = stream
    return p


class Graph:
    """Handle of a ggnn_graph.  Keeps the base tensor alive (the library borrows it)."""

    def __init__(self, handle, base):
        self.h = handle
        self.base = base
        d = GraphDesc()
        _check(lib().ggnn_graph_info(self.h, C.byref(d)))
        self.N, self.D, self.K, self.L, self.s, self.g = d.N, d.D, d.K, d.L, d.s, d.g
        self.dtype, self.metric = d.dtype, d.metric
        self.n = [d.n[l] for l in range(d.L)]
        self.graph_bytes = d.graph_bytes

    def __del__(self):
        try:
            if getattr(self, "h", None) and _lib is not None:
                _lib.ggnn_free(self.h)
                self.h = None
        except Exception:  # interpreter shutdown
            pass

    def info(self):
        d = GraphDesc()
        _check(lib().ggnn_graph_info(self.h, C.byref(d)))
        return d

    # construction steps
    def select(self, l_top):
        _check(lib().ggnn_select(self.h, l_top))

    def merge(self, l_top, l_m):
        _check(lib().ggnn_merge(self.h, l_top, l_m))

    def sym(self, layer):
        _check(lib().ggnn_sym(self.h, layer))

    def build_steps(self):
        _check(lib().ggnn_build_steps(self.h))
        return self

    def set_progress(self, fn):
        """ggnn_build_set_progress: fn(step, l_top, l_m, seconds) after every step of build_steps, or None."""
        if fn is None:
            self._progress = None
            _check(lib().ggnn_build_set_progress(self.h, C.cast(None, ProgressFn), None))
            return
        self._progress = ProgressFn(lambda step, l_top, l_m, seconds, user: fn(step.decode(), l_top, l_m, seconds))
        _check(lib().ggnn_build_set_progress(self.h, self._progress, None))

    def times(self):
        t = BuildTimes()
        _check(lib().ggnn_build_get_times(self.h, C.byref(t)))
        return {k: getattr(t, k) for k, _ in BuildTimes._fields_}

    # host-side access
    def export_layer(self, layer):
        e = np.empty((self.n[layer], self.K), np.int32)
        tl = np.empty(self.n[layer], np.int32) if layer >= 1 else None
        tb = np.empty(self.n[layer], np.int32) if layer >= 1 else None
        _check(lib().ggnn_graph_export(self.h, layer, _host_ptr(e), _host_ptr(tl), _host_ptr(tb)))
        return e, tl, tb

    def import_layer(self, layer, edges=None, to_lower=None, to_base=None):
        conv = lambda a: None if a is None else np.ascontiguousarray(a, np.int32)
        edges, to_lower, to_base = conv(edges), conv(to_lower), conv(to_base)
        _check(lib().ggnn_graph_import(self.h, layer, _host_ptr(edges), _host_ptr(to_lower), _host_ptr(to_base)))

    def export_dnn(self):
        d = np.empty(self.N, np.float32)
        mean, mx = C.c_float(), C.c_float()
        _check(lib().ggnn_graph_export_dnn(self.h, _host_ptr(d), C.byref(mean), C.byref(mx)))
        return d, mean.value, mx.value

    def import_dnn(self, dnn1, mean, mx):
        dnn1 = None if dnn1 is None else np.ascontiguousarray(dnn1, np.float32)
        _check(lib().ggnn_graph_import_dnn(self.h, _host_ptr(dnn1), float(mean), float(mx)))

    def export_inv_count(self, layer):
        c = np.empty(self.n[layer], np.int32)
        _check(lib().ggnn_graph_export_inv_count(self.h, layer, _host_ptr(c)))
        return c

    def query(self, queries, k, beam, slack, pq_cap=0, visited_cap=0, max_iter=0, every_layer=False,
              counters=False, out=None, stream=None, asynchronous=False, start_ids=None, **tuning):
        return query(self, queries, k, beam, slack, pq_cap, visited_cap, max_iter, every_layer, counters, out,
                     stream, asynchronous, start_ids, **tuning)


def query_static(graph, queries, k, beam, slack, out, pq_cap=0, visited_cap=0, max_iter=0, counters=None,
                 stream=None, asynchronous=False):
    """ggnn_query_static: the every-layer search with the library's static workspace.  Nothing is allocated
    here either: `out` = (ids, dists) and, optionally, `counters` (Q x 4 int32) are the caller's tensors."""
    import torch
    _check_query_tensors(graph, queries, k, out, None, counters)
    ids, dists = out
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().ggnn_query_static(graph.h, _dev_ptr(queries), queries.shape[0], k, beam, slack, pq_cap, visited_cap,
                                   max_iter, C.c_void_p(stream), _dev_ptr(ids), _dev_ptr(dists),
                                   _dev_ptr(counters) if counters is not None else None, 1 if asynchronous else 0))
    return ids, dists


def graph_create(base, K, levels, seed=42, metric=L2, segment_size=0, tau_build=0.0, refinements=2, pq_cap=0,
                 visited_cap=0, max_iter=0, sym_constraint=True, stream=None) -> Graph:
    """ggnn_graph_create: an empty graph over `base` (N x D GPU tensor, float32 or uint8)."""
    p = _params(base, metric, segment_size, tau_build, refinements, pq_cap, visited_cap, max_iter, sym_constraint, stream)
    h = C.c_void_p()
    _check(lib().ggnn_graph_create(_dev_ptr(base), base.shape[0], base.shape[1], K, levels, seed, C.byref(p), C.byref(h)))
    return Graph(h, base)


def build(base, K, levels, seed=42, metric=L2, segment_size=0, tau_build=0.0, refinements=2, pq_cap=0,
          visited_cap=0, max_iter=0, sym_constraint=True, stream=None, progress=None) -> Graph:
    """ggnn_build_ex: the whole construction (Alg. 3 followed by r passes of Alg. 6).  With `progress`
    (fn(step, l_top, l_m, seconds)): ggnn_graph_create, ggnn_build_set_progress, ggnn_build_steps."""
    if progress is not None:
        g = graph_create(base, K, levels, seed, metric, segment_size, tau_build, refinements, pq_cap, visited_cap,
                         max_iter, sym_constraint, stream)
        g.set_progress(progress)
        try:
            g.build_steps()
        finally:
            g.set_progress(None)
        return g
    p = _params(base, metric, segment_size, tau_build, refinements, pq_cap, visited_cap, max_iter, sym_constraint, stream)
    h = C.c_void_p()
    _check(lib().ggnn_build_ex(_dev_ptr(base), base.shape[0], base.shape[1], K, levels, seed, C.byref(p), C.byref(h)))
    return Graph(h, base)


def _check_query_tensors(graph, queries, k, out, start_ids, counters=None):
    """The kernels stride the query array by the graph's row length and trust every pointer: shapes, element
    types and devices are checked here, before anything is launched."""
    import torch
    want = torch.uint8 if (graph.dtype == U8 and graph.metric == L2) else torch.float32
    if graph.metric == COSINE and graph.dtype != F32:
        raise TypeError("a cosine graph takes float32 queries")
    if not isinstance(queries, torch.Tensor) or not queries.is_cuda:
        raise TypeError("queries must be a GPU tensor")
    if queries.dim() != 2 or queries.shape[1] != graph.D:
        raise GgnnError("queries must have shape (Q, %d), got %s" % (graph.D, tuple(queries.shape)))
    if queries.dtype != want:
        raise TypeError("queries must be %s like the graph's rows, got %s" % (want, queries.dtype))
    if not queries.is_contiguous():
        raise GgnnError("queries must be contiguous")
    Q = queries.shape[0]
    if k < 1:
        raise GgnnError("k must be positive")
    if out is not None:
        ids, dists = out
        for t, dt, name in ((ids, torch.int32, "ids"), (dists, torch.float32, "dists")):
            if not isinstance(t, torch.Tensor) or t.device != queries.device or t.dtype != dt or tuple(t.shape) != (Q, k) \
                    or not t.is_contiguous():
                raise GgnnError("out %s must be a contiguous %s tensor of shape (%d, %d) on %s" % (name, dt, Q, k, queries.device))
    if counters is not None:
        if not isinstance(counters, torch.Tensor) or counters.device != queries.device or counters.dtype != torch.int32 \
                or tuple(counters.shape) != (Q, 4) or not counters.is_contiguous():
            raise GgnnError("counters must be a contiguous int32 tensor of shape (%d, 4) on %s" % (Q, queries.device))
    if start_ids is not None:
        if not isinstance(start_ids, torch.Tensor) or start_ids.device != queries.device or start_ids.dtype != torch.int32 \
                or start_ids.dim() != 1 or not start_ids.is_contiguous():
            raise GgnnError("start_ids must be a contiguous 1-D int32 tensor on %s" % (queries.device,))


def query(graph, queries, k, beam, slack, pq_cap=0, visited_cap=0, max_iter=0, every_layer=False,
          counters=False, out=None, stream=None, asynchronous=False, start_ids=None, cache_mode=None,
          split_threshold=None, global_visited=None):
    """ggnn_query_ex (ggnn_query_from with start_ids).  Returns (ids, dists[, counters]) as GPU tensors; `out` =
    (ids, dists) reuses buffers.  cache_mode / split_threshold / global_visited: when any is given the call goes
    through ggnn_query_with, which takes them per call instead of from the process-wide defaults."""
    import torch
    _check_query_tensors(graph, queries, k, out, start_ids)
    Q = queries.shape[0]
    if out is None:
        ids = torch.empty((Q, k), dtype=torch.int32, device=queries.device)
        dists = torch.empty((Q, k), dtype=torch.float32, device=queries.device)
    else:
        ids, dists = out
    cnt = torch.zeros((Q, 4), dtype=torch.int32, device=queries.device) if counters else None
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    if cache_mode is not None or split_threshold is not None or global_visited is not None:
        p = QueryParams()
        p.pq_cap, p.visited_cap, p.max_iter, p.every_layer = pq_cap, visited_cap, max_iter, 1 if every_layer else 0
        p.cache_mode = cache_mode or 0
        p.split_min_queries = split_threshold or 0
        p.global_visited_min_iter = global_visited or 0
        p.start_ids_dev = start_ids.data_ptr() if start_ids is not None else None
        p.n_start = start_ids.shape[0] if start_ids is not None else 0
        p.asynchronous, p.stream = (1 if asynchronous else 0), stream
        _check(lib().ggnn_query_with(graph.h, _dev_ptr(queries), Q, k, beam, slack, C.byref(p), _dev_ptr(ids), _dev_ptr(dists),
                                     _dev_ptr(cnt) if counters else None))
        return (ids, dists, cnt) if counters else (ids, dists)
    if start_ids is not None:  # ggnn_query_from: bottom layer only, from the given start points
        _check(lib().ggnn_query_from(graph.h, _dev_ptr(queries), Q, k, beam, slack, pq_cap, visited_cap, max_iter,
                                     _dev_ptr(start_ids), start_ids.shape[0], C.c_void_p(stream), _dev_ptr(ids),
                                     _dev_ptr(dists), _dev_ptr(cnt) if counters else None, 1 if asynchronous else 0))
        return (ids, dists, cnt) if counters else (ids, dists)
    _check(lib().ggnn_query_ex(graph.h, _dev_ptr(queries), Q, k, beam, slack, pq_cap, visited_cap, max_iter,
                               1 if every_layer else 0, C.c_void_p(stream), _dev_ptr(ids), _dev_ptr(dists),
                               _dev_ptr(cnt) if counters else None, 1 if asynchronous else 0))
    return (ids, dists, cnt) if counters else (ids, dists)
