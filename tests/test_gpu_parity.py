"""GPU parity tests: the HIP library against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


@pytest.fixture(scope="module", params=["registers", "lds"])
def ggnn(request):
    """The library, once with best / prioq in registers (when they fit) and once forced into LDS."""
    _need_gpu()
    import paper_1912_01059_amd as m
    m.lib()
    m.set_cache_mode(1 if request.param == "lds" else 0)
    yield m
    m.set_cache_mode(0)


@pytest.fixture(scope="module")
def R():
    from oracle import ggnn_ref
    return ggnn_ref


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_gpu_graph(ggnn, og, base_t, **kw):
    """Loads the state of an oracle graph into a library graph over the same base."""
    g = ggnn.graph_create(base_t, og.K, og.L, seed=og.seed, metric=og.metric, segment_size=og.s, **kw)
    for l in range(og.L):
        g.import_layer(l, og.edges(l), og.to_lower(l) if l >= 1 else None, og.to_base(l) if l >= 1 else None)
    st = og.stats()
    g.import_dnn(og.dnn1(), float(st[0]), float(st[1]))
    return g


def assert_same_results(got_ids, got_d, want_ids, want_d):
    got_ids, got_d = got_ids.cpu().numpy(), got_d.cpu().numpy()
    assert np.array_equal(got_ids, want_ids)
    assert np.array_equal(got_d.view(np.uint32), want_d.view(np.uint32))  # bit for bit


def check_counters(cnt, rcnt):
    """pops and the method's distance evaluations are those of the oracle; the rows actually
    gathered are fewer (re-evaluations of rejected points are skipped)."""
    c = cnt.cpu().numpy().astype(np.uint32)
    assert np.array_equal(c[:, :2], rcnt)
    assert (c[:, 2] <= c[:, 1]).all()


# ------------------------------------------------------------------------------ query

@pytest.mark.parametrize("every_layer", [False, True])
@pytest.mark.parametrize("k,beam,tau", [(10, 10, 0.0), (10, 10, 0.3), (10, 64, 0.5), (1, 10, 0.4), (24, 24, 0.2),
                                         (100, 100, 0.3), (10, 128, 0.1), (70, 65, 0.2), (130, 130, 0.2)])
def test_query_matches_oracle_on_config1(ggnn, R, sift10k, sift10k_oracle_graph, every_layer, k, beam, tau):
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    g = to_gpu_graph(ggnn, og, dev(base))
    ids, d, cnt = g.query(dev(queries), k, beam, tau, visited_cap=384, every_layer=every_layer, counters=True)
    rids, rd, rcnt = og.query(queries, k, beam, tau, visited_cap=384, every_layer=every_layer, counters=True)
    assert_same_results(ids, d, rids, rd)
    check_counters(cnt, rcnt)


def test_query_small_capacities_and_iteration_limit(ggnn, R, sift10k, sift10k_oracle_graph):
    """prioq overflow, visited limit and iteration limit behave as in the oracle."""
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    g = to_gpu_graph(ggnn, og, dev(base))
    q = dev(queries[:300])
    for P, V, it in [(4, 16, 16), (8, 64, 10), (100, 500, 500), (64, 384, 1), (64, 5000, 5000), (100, 9000, 9000), (64, 385, 385), (32, 777, 700)]:
        ids, d, cnt = g.query(q, 10, 10, 0.4, pq_cap=P, visited_cap=V, max_iter=it, every_layer=True, counters=True)
        rids, rd, rcnt = og.query(queries[:300], 10, 10, 0.4, pq_cap=P, visited_cap=V, max_iter=it, every_layer=True,
                                  counters=True)
        assert_same_results(ids, d, rids, rd)
        check_counters(cnt, rcnt)


def test_query_exhaustive_beam_equals_brute_force(ggnn, R):
    """best as long as the data set: the whole reachable set is visited; on a connected graph
    that is the exact answer."""
    rng = np.random.default_rng(5)
    N, D, K = 200, 16, 12
    base = rng.standard_normal((N, D)).astype(np.float32)
    og = R.Graph(base, K, 2, seed=3).build()
    g = to_gpu_graph(ggnn, og, dev(base))
    q = rng.standard_normal((64, D)).astype(np.float32)
    ids, d = g.query(dev(q), 10, N, 0.0, pq_cap=N, visited_cap=N, max_iter=N)
    rids, rd = og.query(q, 10, N, 0.0, pq_cap=N, visited_cap=N, max_iter=N)
    assert_same_results(ids, d, rids, rd)
    gt_ids, gt_d = R.bruteforce(base, q, 10)
    assert np.array_equal(ids.cpu().numpy(), gt_ids)


def test_query_real_valued_data_bit_exact(ggnn, R):
    """Real-valued rows (D=96, unit length): the fixed float32 summation order makes the
    traversal identical to the oracle's, not merely close."""
    import ggnn_inputs
    base, queries, cfg = ggnn_inputs.make("deep1m", n=6000, q=400)
    og = R.Graph(base, 24, 3, seed=9).build()
    g = to_gpu_graph(ggnn, og, dev(base))
    for every_layer in (False, True):
        ids, d, cnt = g.query(dev(queries), 10, 10, 0.4, every_layer=every_layer, counters=True)
        rids, rd, rcnt = og.query(queries, 10, 10, 0.4, every_layer=every_layer, counters=True)
        assert_same_results(ids, d, rids, rd)
        check_counters(cnt, rcnt)
    # and within 1e-5 relative of float64 distances
    b64, q64 = base.astype(np.float64), queries.astype(np.float64)
    got = ids.cpu().numpy()
    for i in range(0, 400, 13):
        ref = np.sqrt(((b64[got[i]] - q64[i]) ** 2).sum(1))
        assert np.allclose(d.cpu().numpy()[i], ref, rtol=1e-5, atol=0)


def test_query_cosine_matches_oracle(ggnn, R):
    import ggnn_inputs
    base, queries, cfg = ggnn_inputs.make("glove1m", n=5000, q=300)
    og = R.Graph(base, 40, 3, metric=R.COSINE, seed=4).build()
    g = to_gpu_graph(ggnn, og, dev(base))
    ids, d = g.query(dev(queries), 10, 10, 0.5, visited_cap=512, every_layer=True)
    rids, rd = og.query(queries, 10, 10, 0.5, visited_cap=512, every_layer=True)
    assert_same_results(ids, d, rids, rd)


def test_query_uint8_matches_oracle(ggnn, R):
    import ggnn_inputs
    base, queries, cfg = ggnn_inputs.make("sift100m_u8", n=5000, q=300)
    assert base.dtype == np.uint8
    og = R.Graph(base, 24, 3, seed=4).build()
    g = to_gpu_graph(ggnn, og, dev(base))
    ids, d = g.query(dev(queries), 10, 10, 0.3, every_layer=True)
    rids, rd = og.query(queries, 10, 10, 0.3, every_layer=True)
    assert_same_results(ids, d, rids, rd)


def test_query_edge_cases(ggnn, R, sift10k, sift10k_oracle_graph):
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    g = to_gpu_graph(ggnn, og, dev(base))
    # no queries
    ids, d = g.query(dev(queries[:0]), 10, 10, 0.3)
    assert ids.shape == (0, 10)
    # one query, ragged sizes
    for Q in (1, 63, 65):
        ids, d = g.query(dev(queries[:Q]), 10, 10, 0.3)
        rids, rd = og.query(queries[:Q], 10, 10, 0.3)
        assert_same_results(ids, d, rids, rd)
    # invalid arguments are errors, not faults
    with pytest.raises(ggnn.GgnnError):
        g.query(dev(queries[:4]), 0, 10, 0.3)
    with pytest.raises(ggnn.GgnnError):
        g.query(dev(queries[:4]), 10, 10, -1.0)
    with pytest.raises(ggnn.GgnnError):
        g.query(dev(queries[:4]), 10, 10, 0.3, visited_cap=100, max_iter=200)
    with pytest.raises(ggnn.GgnnError):
        g.query(dev(queries[:4]), 10, 4000, 0.3, pq_cap=4000, visited_cap=20000)  # over the LDS budget
    bad = og.edges(0).copy()
    bad[5, 3] = bad[5, 2]
    with pytest.raises(ggnn.GgnnError):
        g.import_layer(0, bad)
    bad = og.edges(0).copy()
    bad[7, 0] = 10_000
    with pytest.raises(ggnn.GgnnError):
        g.import_layer(0, bad)


# ------------------------------------------------------------------------------ construction steps

def test_merge_select_stats_match_oracle_step_by_step(ggnn, R, sift10k):
    """Every deterministic construction step, run on the state the oracle reached so far."""
    base, _, cfg = sift10k
    K, L = cfg["K"], cfg["levels"]
    og = R.Graph(base, K, L, seed=42)
    g = ggnn.graph_create(dev(base), K, L, seed=42)
    assert g.n == og.n and g.g == og.g
    p = R.default_params()

    def sync_from_oracle():
        for l in range(L):
            e = og.edges(l)
            if (e >= 0).any() or l == 0:
                g.import_layer(l, e, og.to_lower(l) if l >= 1 else None, og.to_base(l) if l >= 1 else None)
        st = og.stats()
        g.import_dnn(og.dnn1(), float(st[0]), float(st[1]))

    def check_layer(l):
        e, tl, tb = g.export_layer(l)
        assert np.array_equal(e, og.edges(l)), "edges of layer %d" % l
        if l >= 1:
            assert np.array_equal(tl, og.to_lower(l)) and np.array_equal(tb, og.to_base(l))

    def check_dnn():
        d, mean, mx = g.export_dnn()
        assert np.array_equal(d.view(np.uint32), og.dnn1().view(np.uint32))
        assert mx == og.stats()[1]
        assert abs(mean - og.stats()[0]) <= 2 ** -22 * mean

    # merge(0,0): exhaustive search inside the bottom segments, then stats
    og.merge(0, 0, p); g.merge(0, 0); check_layer(0); check_dnn()
    og.sym(0, p); sync_from_oracle()
    for l_top in range(1, L):
        og.select(l_top); g.select(l_top)
        e, tl, tb = g.export_layer(l_top)
        assert np.array_equal(tl, og.to_lower(l_top)) and np.array_equal(tb, og.to_base(l_top))
        for l_m in range(l_top, -1, -1):
            og.merge(l_top, l_m, p); g.merge(l_top, l_m); check_layer(l_m)
            if l_m == 0:
                check_dnn()
            og.sym(l_m, p); sync_from_oracle()


def test_sym_matches_oracle(ggnn, R, sift10k):
    base, _, cfg = sift10k
    K, L = cfg["K"], cfg["levels"]
    og = R.Graph(base, K, L, seed=42)
    g = ggnn.graph_create(dev(base), K, L, seed=42)
    p = R.default_params()
    og.merge(0, 0, p)
    g.import_layer(0, og.edges(0))
    st = og.stats()
    g.import_dnn(og.dnn1(), float(st[0]), float(st[1]))
    og.sym(0, p)
    g.sym(0)
    e, _, _ = g.export_layer(0)
    assert np.array_equal(g.export_inv_count(0), og.inv_count(0))
    assert np.array_equal(e, og.edges(0))


def test_full_build_matches_oracle(ggnn, R, sift10k, sift10k_oracle_graph):
    """The whole construction on config 1 gives the oracle's graph, layer by layer."""
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    g = ggnn.build(dev(base), cfg["K"], cfg["levels"], seed=42)
    for l in range(g.L):
        e, tl, tb = g.export_layer(l)
        assert np.array_equal(e, og.edges(l)), "layer %d" % l
        if l >= 1:
            assert np.array_equal(tl, og.to_lower(l)) and np.array_equal(tb, og.to_base(l))
    t = g.times()
    assert t["total_ms"] > 0 and t["merge_ms"] > 0 and t["sym_ms"] > 0


def test_build_quality_and_recall(ggnn, R, sift10k, sift10k_gt):
    """Invariants of a GPU-built graph and recall against exhaustive search (config 1)."""
    base, queries, cfg = sift10k
    K = cfg["K"]
    g = ggnn.build(dev(base), K, cfg["levels"], seed=7)
    e0, _, _ = g.export_layer(0)
    assert (e0 >= 0).all()
    srt = np.sort(e0, axis=1)
    assert (np.diff(srt, axis=1) > 0).all()                      # distinct
    assert not (e0 == np.arange(len(e0))[:, None]).any()         # no self loop
    assert g.export_inv_count(0).max() <= K - K // 2
    ids, _ = g.query(dev(queries), 10, 10, 0.3, every_layer=True)
    assert R.recall(ids.cpu().numpy(), sift10k_gt[0]) >= 0.99


# ------------------------------------------------------------------------------ construction, varied shapes

@pytest.mark.parametrize("case", [
    dict(N=200, D=16, K=12, L=2, s=32, kind="real"),            # tiny, one bottom segment per 32 points
    dict(N=777, D=8, K=6, L=3, s=16, kind="int"),               # ragged segments, small s
    dict(N=2000, D=32, K=40, L=3, s=32, kind="int"),            # K above the segment size: rows padded with -1 at first
    dict(N=1500, D=100, K=24, L=2, s=32, kind="cosine"),        # cosine, D not a multiple of 32
    dict(N=3000, D=128, K=24, L=3, s=32, kind="u8"),            # uint8 rows
    dict(N=1200, D=96, K=25, L=3, s=32, kind="real"),           # odd K: k_nn = 12, k_sym = 13
    dict(N=890, D=64, K=24, L=2, s=64, kind="dups"),            # duplicated rows: distance ties, zero distances
    dict(N=1500, D=960, K=24, L=2, s=32, kind="real"),          # rows above 1024 bytes: 64 lanes per row, ragged last chunk
    dict(N=1200, D=320, K=24, L=3, s=32, kind="real"),          # 64 lanes per row, two chunks per lane, second one partly filled
    dict(N=1000, D=300, K=24, L=2, s=32, kind="cosine"),        # cosine on rows above 1024 bytes
    dict(N=900, D=1024, K=16, L=2, s=32, kind="int"),           # the longest float32 row
    dict(N=1000, D=256, K=24, L=2, s=32, kind="u8"),            # the longest uint8 row
    dict(N=1000, D=256, K=24, L=2, s=32, kind="real"),          # the longest float32 row with 8 lanes per row
    dict(N=3000, D=16, K=64, L=2, s=64, kind="int"),            # the largest out-degree and segment size
    dict(N=4000, D=8, K=8, L=5, s=8, kind="real"),              # five levels of small segments
])
def test_full_build_matches_oracle_on_varied_shapes(ggnn, R, case):
    rng = np.random.default_rng(case["N"])
    N, D = case["N"], case["D"]
    metric_o, metric_g = R.L2, ggnn.L2
    if case["kind"] in ("real", "cosine"):
        base = rng.standard_normal((N, D)).astype(np.float32)
        if case["kind"] == "cosine":
            base *= np.exp(rng.normal(0, 0.5, (N, 1))).astype(np.float32)
            metric_o, metric_g = R.COSINE, ggnn.COSINE
    elif case["kind"] == "u8":
        base = rng.integers(0, 256, (N, D)).astype(np.uint8)
    else:
        base = rng.integers(0, 256, (N, D)).astype(np.float32)
        if case["kind"] == "dups":
            base[N // 2:] = base[: N - N // 2]
    p = R.default_params(refinements=1, visited_cap=96, max_iter=96)
    og = R.Graph(base, case["K"], case["L"], s=case["s"], metric=metric_o, seed=5).build(p)
    g = ggnn.build(dev(base), case["K"], case["L"], seed=5, metric=metric_g, segment_size=case["s"], refinements=1,
                   visited_cap=96, max_iter=96)
    assert g.n == og.n
    for l in range(g.L):
        e, tl, tb = g.export_layer(l)
        assert np.array_equal(e, og.edges(l)), "layer %d" % l
        if l >= 1:
            assert np.array_equal(tl, og.to_lower(l)) and np.array_equal(tb, og.to_base(l))
        assert np.array_equal(g.export_inv_count(l), og.inv_count(l))
    d, mean, mx = g.export_dnn()
    assert np.array_equal(d.view(np.uint32), og.dnn1().view(np.uint32)) and mx == og.stats()[1]
    # queries on it, both descent modes, results padded when fewer than k points are reachable
    q = base[rng.integers(0, N, 50)].copy()
    for every in (False, True):
        ids, dd = g.query(dev(q), 10, 10, 0.3, every_layer=every)
        rids, rd = og.query(q, 10, 10, 0.3, every_layer=every)
        assert_same_results(ids, dd, rids, rd)


# ------------------------------------------------------------------------------ shards

def test_shard_merge_matches_oracle(ggnn, R):
    rng = np.random.default_rng(8)
    for S, Q, k in [(1, 5, 3), (4, 130, 10), (7, 64, 100), (16, 33, 1)]:
        d = np.sort(rng.integers(0, 50, (S, Q, k)).astype(np.float32), axis=2)     # many ties across shards
        ids = np.stack([np.stack([rng.choice(1000, k, replace=False) for _ in range(Q)]) for _ in range(S)]).astype(np.int32)
        pad = rng.random((S, Q)) < 0.3
        for s in range(S):
            for q in range(Q):
                if pad[s, q]:
                    cut = int(rng.integers(0, k + 1))
                    ids[s, q, cut:] = -1
                    d[s, q, cut:] = np.inf
        offsets = (np.arange(S) * 1000).astype(np.int32)
        gi, gd = ggnn.merge_shards(dev(ids), dev(d), dev(offsets))
        ri, rd = R.merge_shards(ids, d, offsets)
        assert np.array_equal(gi.cpu().numpy(), ri) and np.array_equal(gd.cpu().numpy().view(np.uint32), rd.view(np.uint32))


def test_sharded_index_recall(ggnn, R, sift10k, sift10k_gt):
    """Four shards of config 1, each with its own graph: merged answers against exhaustive search."""
    base, queries, cfg = sift10k
    idx = ggnn.ShardedIndex(dev(base), 4, cfg["K"], 3, seed=3)
    ids, d = idx.query(dev(queries), 10, 10, 0.3, every_layer=True)
    assert R.recall(ids.cpu().numpy(), sift10k_gt[0]) >= 0.99
    got = ids.cpu().numpy()
    d2 = ((base[got[0]].astype(np.int64) - queries[0].astype(np.int64)) ** 2).sum(1)
    assert np.array_equal(d.cpu().numpy()[0], np.sqrt(d2.astype(np.float32)))


# ------------------------------------------------------------------------------ explicit start points

def test_query_from_start_points(ggnn, R, sift10k, sift10k_oracle_graph):
    """Centroid / worst-point starts of the paper's appendix on config 1, and argument checks."""
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    g = to_gpu_graph(ggnn, og, dev(base))
    centre = base.mean(0)
    d2 = ((base - centre) ** 2).sum(1)
    for starts in (np.array([d2.argmin()], np.int32), np.array([d2.argmax()], np.int32),
                   np.arange(0, 6400, 100, dtype=np.int32)):
        ids, d = g.query(dev(queries), 10, 10, 0.4, start_ids=dev(starts))
        rids, rd = og.query(queries, 10, 10, 0.4, start_ids=starts)
        assert_same_results(ids, d, rids, rd)
    with pytest.raises(ggnn.GgnnError):
        g.query(dev(queries[:4]), 10, 10, 0.4, start_ids=dev(np.array([5, 5], np.int32)))
    with pytest.raises(ggnn.GgnnError):
        g.query(dev(queries[:4]), 10, 10, 0.4, start_ids=dev(np.array([10_000], np.int32)))
    with pytest.raises(ggnn.GgnnError):
        g.query(dev(queries[:4]), 10, 10, 0.4, start_ids=dev(np.arange(65, dtype=np.int32)))


# ------------------------------------------------------------------------------ large batches in two launches

def test_two_launch_path_matches_one_launch_and_oracle(ggnn, R, sift10k, sift10k_oracle_graph):
    """Large batches are answered in two launches (upper layers; bottom layer in an order sorted by
    region, one part per XCD).  Forced here for small batches: results and counters must be those of
    the one-launch path and of the oracle."""
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    g = to_gpu_graph(ggnn, og, dev(base))
    rng = np.random.default_rng(3)
    for Q, k, beam, tau, P in [(997, 10, 10, 0.3, 64), (1000, 10, 100, 0.2, 64), (8, 5, 16, 0.5, 32), (3, 1, 1, 0.0, 64)]:
        q = queries[rng.integers(0, len(queries), Q)].copy()
        ids1, d1, c1 = g.query(dev(q), k, beam, tau, pq_cap=P, every_layer=True, counters=True)
        ggnn.set_split_threshold(1)
        try:
            ids2, d2, c2 = g.query(dev(q), k, beam, tau, pq_cap=P, every_layer=True, counters=True)
        finally:
            ggnn.set_split_threshold(0)
        assert torch.equal(ids1, ids2) and torch.equal(d1.view(torch.int32), d2.view(torch.int32))
        assert torch.equal(c1, c2)
        rids, rd, rcnt = og.query(q, k, beam, tau, pq_cap=P, every_layer=True, counters=True)
        assert_same_results(ids2, d2, rids, rd)
        check_counters(c2, rcnt)


# ------------------------------------------------------------------------------ visited set in global memory

def test_global_visited_table_matches_lds_table_and_oracle(ggnn, R, sift10k, sift10k_oracle_graph):
    """Long searches keep the visited ids in a per-query table in global memory instead of LDS.  Forced
    here for short ones too: results and the method's counters (pops, distance evaluations) must be
    those of the LDS table and of the oracle, in both descent modes, for both best-list widths, with
    explicit start points, and on cosine and uint8 data."""
    import ggnn_inputs
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    g = to_gpu_graph(ggnn, og, dev(base))
    rng = np.random.default_rng(5)
    cases = [(500, 10, 10, 0.3, 64, 384, True), (300, 10, 100, 0.2, 64, 200, False), (64, 24, 24, 1.0, 32, 1500, True),
             (5, 1, 1, 0.0, 64, 1, True), (200, 100, 128, 0.4, 64, 3000, True)]
    for Q, k, beam, tau, P, V, every in cases:
        q = queries[rng.integers(0, len(queries), Q)].copy()
        kw = dict(pq_cap=P, visited_cap=V, max_iter=V, every_layer=every, counters=True)
        ggnn.set_global_visited_threshold(-1)
        try:
            ids1, d1, c1 = g.query(dev(q), k, beam, tau, **kw)
            ggnn.set_global_visited_threshold(1)
            ids2, d2, c2 = g.query(dev(q), k, beam, tau, **kw)
        finally:
            ggnn.set_global_visited_threshold(0)
        assert torch.equal(ids1, ids2) and torch.equal(d1.view(torch.int32), d2.view(torch.int32))
        assert torch.equal(c1[:, :2], c2[:, :2])
        rids, rd, rcnt = og.query(q, k, beam, tau, pq_cap=P, visited_cap=V, max_iter=V, every_layer=every, counters=True)
        assert_same_results(ids2, d2, rids, rd)
        check_counters(c2, rcnt)
    # explicit start points on the bottom layer
    starts = np.arange(0, 3200, 100, dtype=np.int32)
    ggnn.set_global_visited_threshold(1)
    try:
        ids, d, c = g.query(dev(queries[:200]), 10, 16, 0.5, visited_cap=256, counters=True, start_ids=dev(starts))
    finally:
        ggnn.set_global_visited_threshold(0)
    rids, rd, rcnt = og.query(queries[:200], 10, 16, 0.5, visited_cap=256, counters=True, start_ids=starts)
    assert_same_results(ids, d, rids, rd)
    check_counters(c, rcnt)
    # other element types and metrics
    for name, n, nq in (("glove1m", 4000, 200), ("deep1m", 4000, 200)):
        b2, q2, c2cfg = ggnn_inputs.make(name, n=n, q=nq)
        metric_o = R.COSINE if c2cfg["metric"] == "cosine" else R.L2
        og2 = R.Graph(b2, c2cfg["K"], 3, metric=metric_o, seed=7).build(R.default_params(visited_cap=96, max_iter=96))
        g2 = to_gpu_graph(ggnn, og2, dev(b2))
        ggnn.set_global_visited_threshold(1)
        try:
            ids, d, c = g2.query(dev(q2), 10, 10, 0.4, visited_cap=700, every_layer=True, counters=True)
        finally:
            ggnn.set_global_visited_threshold(0)
        rids, rd, rcnt = og2.query(q2, 10, 10, 0.4, visited_cap=700, every_layer=True, counters=True)
        assert_same_results(ids, d, rids, rd)
        check_counters(c, rcnt)
    b3 = np.random.default_rng(9).integers(0, 256, (3000, 64)).astype(np.uint8)
    q3 = np.random.default_rng(10).integers(0, 256, (150, 64)).astype(np.uint8)
    og3 = R.Graph(b3, 24, 3, seed=7).build(R.default_params(visited_cap=96, max_iter=96))
    g3 = to_gpu_graph(ggnn, og3, dev(b3))
    ggnn.set_global_visited_threshold(1)
    try:
        ids, d, c = g3.query(dev(q3), 10, 10, 0.6, visited_cap=600, every_layer=True, counters=True)
    finally:
        ggnn.set_global_visited_threshold(0)
    rids, rd, rcnt = og3.query(q3, 10, 10, 0.6, visited_cap=600, every_layer=True, counters=True)
    assert_same_results(ids, d, rids, rd)
    check_counters(c, rcnt)


# ------------------------------------------------------------------------------ capture into a HIP graph

def test_query_replayed_from_a_hip_graph(ggnn, R, sift10k, sift10k_oracle_graph):
    """A batch below the two-launch threshold is one kernel launch and no allocation, so it can be
    captured into a HIP graph: every replay, with eager work and synchronisations in between and new
    queries in the captured input buffer, gives the oracle's answers."""
    base, queries, cfg = sift10k
    og = sift10k_oracle_graph
    g = to_gpu_graph(ggnn, og, dev(base))
    Q, k = 256, 10
    qbuf = dev(queries[:Q].copy())
    ids = torch.empty((Q, k), dtype=torch.int32, device="cuda")
    d = torch.empty((Q, k), dtype=torch.float32, device="cuda")
    g.query(qbuf, k, 10, 0.3, every_layer=True, out=(ids, d))  # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        g.query(qbuf, k, 10, 0.3, every_layer=True, out=(ids, d), asynchronous=True)
    for rep in range(4):
        part = queries[rep * 150: rep * 150 + Q].copy()
        qbuf.copy_(dev(part))
        ids.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        rids, rd = og.query(part, k, 10, 0.3, every_layer=True)
        assert_same_results(ids, d, rids, rd)
        eager_ids, eager_d = g.query(qbuf, k, 10, 0.3, every_layer=True)  # eager work between the replays
        assert torch.equal(eager_ids, ids)
