"""MI355X (gfx950) implementation of GGNN's hot path: batched best-first search over a
hierarchical kNN graph and the graph construction driven by it.  Thin ctypes binding of
libggnn.so; PyTorch is used only for device memory and streams."""
from .binding import (  # noqa: F401
    COSINE, F32, L2, U8, BuildParams, QueryParams, Graph, GgnnError, ShardedIndex, build, gather_probe, graph_create, merge_shards, last_error, lib, query, query_static, set_cache_mode, set_global_visited_threshold, set_split_threshold,
)
