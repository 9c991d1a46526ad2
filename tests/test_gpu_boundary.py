"""The C ABI's plain entry points with real data, straight through ctypes: ggnn_build and ggnn_query at their
documented defaults against the oracle, ggnn_graph_info against the sizes the paper prints, and
ggnn_query_with against ggnn_query_ex."""
import ctypes as C
import os

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
HERE = os.path.dirname(os.path.abspath(__file__))


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def test_plain_build_and_query_use_the_documented_defaults(sift10k, sift10k_oracle_graph):
    """ggnn_build(base, N, D, K, levels, seed) and ggnn_query(g, q, Q, k, beam, slack) as the header declares
    them: float32, L2, s = 32, tau_b = 0.5, two refinement passes, construction cache 64 / 384; query cache
    prioq 64, visited 384 (896 from a best list of 100), iteration limit = visited, top layer then bottom
    layer.  Graph and answers must be the oracle's at the same settings, bit for bit."""
    _need_gpu()
    from paper_1912_01059_amd import binding
    L = binding.lib()
    L.ggnn_set_cache_mode(0)
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    b = torch.from_numpy(base).cuda()
    q = torch.from_numpy(queries).cuda()
    h = C.c_void_p()
    rc = L.ggnn_build(C.c_void_p(b.data_ptr()), base.shape[0], base.shape[1], cfg["K"], cfg["levels"], 42, C.byref(h))
    assert rc == 0, L.ggnn_last_error()
    try:
        for l in range(cfg["levels"]):
            e = np.empty((og.n[l], cfg["K"]), np.int32)
            assert L.ggnn_graph_export(h, l, e.ctypes.data_as(C.c_void_p), None, None) == 0
            assert np.array_equal(e, og.edges(l)), "layer %d" % l
        for k, beam, visited in [(10, 10, 384), (10, 64, 384), (100, 100, 896)]:
            ids = torch.empty((len(queries), k), dtype=torch.int32, device="cuda")
            d = torch.empty((len(queries), k), dtype=torch.float32, device="cuda")
            rc = L.ggnn_query(h, C.c_void_p(q.data_ptr()), len(queries), k, beam, 0.3, C.c_void_p(ids.data_ptr()),
                              C.c_void_p(d.data_ptr()))
            assert rc == 0, L.ggnn_last_error()
            rids, rd = og.query(queries, k, beam, 0.3, pq_cap=64, visited_cap=visited, every_layer=False)
            assert np.array_equal(ids.cpu().numpy(), rids)
            assert np.array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))
    finally:
        L.ggnn_free(h)


def test_graph_info_gives_the_sizes_the_paper_prints():
    """Appendix 'Graph Size' / Table 4, from tests/golden/graph_size.txt: one million points, s = 32, four layers
    give g = 32 and 33 824 upper-layer points; the graph takes 94.9 MiB at K = 24 and 158 MiB at K = 40."""
    _need_gpu()
    import paper_1912_01059_amd as ggnn
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "graph_size.txt")) if l.strip() and not l.startswith("#")]
    base = torch.zeros((1_000_000, 16), dtype=torch.float32, device="cuda")
    checked = 0
    for row in rows:
        N, s, L, K, g_exp, n_upper = (int(v) for v in row[:6])
        if N != 1_000_000:
            continue
        g = ggnn.graph_create(base, K, L, segment_size=s)
        d = g.info()
        assert d.g == g_exp and sum(d.n[l] for l in range(1, L)) == n_upper and d.n[0] == N and d.n[L - 1] == s
        assert abs(d.graph_bytes / 2 ** 20 - float(row[6])) <= float(row[7])
        checked += 1
    assert checked == 2


def test_per_call_parameters_give_the_results_of_the_process_wide_ones(sift10k):
    """ggnn_query_with: cache placement, two-launch threshold and visited placement passed per call -- every
    combination answers as ggnn_query_ex does (results and the method's counters do not depend on them)."""
    _need_gpu()
    import paper_1912_01059_amd as ggnn
    ggnn.set_cache_mode(0)
    base, queries, cfg = sift10k
    b = torch.from_numpy(base).cuda()
    q = torch.from_numpy(queries[:600]).cuda()
    g = ggnn.build(b, cfg["K"], cfg["levels"], seed=42, visited_cap=96, max_iter=96)
    for every in (True, False):
        want_ids, want_d, want_c = g.query(q, 10, 16, 0.3, visited_cap=200, every_layer=every, counters=True)
        for kw in (dict(cache_mode=1), dict(split_threshold=1), dict(global_visited=1), dict(split_threshold=-1, global_visited=-1),
                   dict(cache_mode=0, split_threshold=1, global_visited=1)):
            ids, d, c = g.query(q, 10, 16, 0.3, visited_cap=200, every_layer=every, counters=True, **kw)
            assert torch.equal(ids, want_ids), kw
            assert torch.equal(d.view(torch.int32), want_d.view(torch.int32)), kw
            assert torch.equal(c[:, :2], want_c[:, :2]), kw
    starts = torch.arange(0, 3200, 100, dtype=torch.int32, device="cuda")
    a = g.query(q, 10, 16, 0.5, start_ids=starts)
    bq = g.query(q, 10, 16, 0.5, start_ids=starts, global_visited=1)
    assert torch.equal(a[0], bq[0]) and torch.equal(a[1].view(torch.int32), bq[1].view(torch.int32))


def test_progress_callback_reports_every_step_of_the_construction(sift10k):
    """ggnn_build_set_progress: the callback sees the steps of Alg. 3 (select, then merge and symmetric linking
    from the new top layer down to the bottom) followed by the refinement passes of Alg. 6, in order, with
    non-decreasing times; the graph is the one the plain construction gives, and a later step-wise call still
    works after ggnn_build_steps has returned its construction buffers."""
    _need_gpu()
    import paper_1912_01059_amd as ggnn
    base, queries, cfg = sift10k
    b = torch.from_numpy(base).cuda()
    L_, r = cfg["levels"], 2
    seen = []
    g = ggnn.build(b, cfg["K"], L_, seed=42, refinements=r, visited_cap=96, max_iter=96,
                   progress=lambda step, l_top, l_m, seconds: seen.append((step, l_top, l_m, seconds)))
    want = []
    for l_top in range(L_):
        if l_top > 0:
            want.append(("select", l_top, -1))
        for l_m in range(l_top, -1, -1):
            want += [("merge", l_top, l_m), ("sym", -1, l_m)]
    for _ in range(r):
        for l_m in range(L_ - 2, -1, -1):
            want += [("merge", L_ - 1, l_m), ("sym", -1, l_m)]
    assert [s[:3] for s in seen] == want
    times = [s[3] for s in seen]
    assert all(t1 >= t0 >= 0.0 for t0, t1 in zip(times, times[1:]))
    plain = ggnn.build(b, cfg["K"], L_, seed=42, refinements=r, visited_cap=96, max_iter=96)
    for l in range(L_):
        for x, y in zip(g.export_layer(l), plain.export_layer(l)):
            assert (x is None and y is None) or np.array_equal(x, y)
    assert g.times()["merge_pops"] == plain.times()["merge_pops"] > 0
    n_seen = len(seen)
    g.sym(0)  # allocates the construction buffers again; no callback outside ggnn_build_steps
    assert len(seen) == n_seen
