"""GPU-vs-oracle search parity on many small random graphs: arbitrary (valid) adjacency rows with
-1 padding, random translation tables, random cache capacities, both descent modes, integer- and
real-valued rows.  Nothing here is a kNN graph: the state machine itself is what is compared."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _random_case(seed):
    from oracle import ggnn_ref as R
    rng = np.random.default_rng(seed)
    while True:
        N = int(rng.integers(70, 700))
        s = int(rng.choice([8, 16, 32]))
        L = int(rng.choice([2, 3]))
        try:
            g, n, G = R.geometry(N, s, L)
        except ValueError:
            continue
        if -(-N // G[0]) > 64:
            continue
        break
    D = int(rng.choice([4, 8, 20, 32, 100, 128]))
    K = int(rng.integers(2, 33))
    real = bool(rng.integers(0, 2))
    base = rng.standard_normal((N, D)).astype(np.float32) if real else rng.integers(0, 256, (N, D)).astype(np.float32)
    if not real and rng.integers(0, 2):
        base[rng.integers(0, N, 5)] = base[rng.integers(0, N, 5)]  # exact duplicates: distance ties
    layers = []
    for l in range(L):
        nl = n[l]
        rows = np.full((nl, K), -1, np.int32)
        for i in range(nl):
            cnt = int(rng.integers(0, min(K, nl - 1) + 1)) if rng.random() < 0.3 else min(K, nl - 1)
            cand = rng.choice(nl - 1, cnt, replace=False)
            cand[cand >= i] += 1
            rows[i, :cnt] = cand
        layers.append(rows)
    to_lower, to_base = [None], [None]
    prev_base = np.arange(N)
    for l in range(1, L):
        tl = rng.choice(n[l - 1], n[l], replace=False).astype(np.int32)
        to_lower.append(tl)
        to_base.append(prev_base[tl].astype(np.int32))
        prev_base = to_base[l]
    Q = int(rng.integers(1, 90))
    if real:
        queries = rng.standard_normal((Q, D)).astype(np.float32)
    else:
        queries = rng.integers(0, 256, (Q, D)).astype(np.float32)
        queries[: Q // 3] = base[rng.integers(0, N, Q // 3)]  # queries that coincide with base rows
    k = int(rng.integers(1, 20))
    beam = int(rng.integers(1, 70)) if rng.random() < 0.6 else int(rng.integers(65, 140))
    P = int(rng.integers(1, 80)) if rng.random() < 0.8 else int(rng.integers(80, 200))
    V = int(rng.integers(1, 300))
    it = int(rng.integers(1, V + 1))
    tau = float(rng.choice([0.0, 0.1, 0.5, 1.5]))
    stats = (float(rng.uniform(0.1, 50.0)), float(rng.uniform(50.0, 500.0)))
    return dict(N=N, s=s, L=L, K=K, D=D, base=base, layers=layers, to_lower=to_lower, to_base=to_base,
                queries=queries, k=k, beam=beam, P=P, V=V, it=it, tau=tau, stats=stats, seed=seed)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("seed", range(40))
def test_search_matches_oracle_on_random_graph(seed, mode):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1912_01059_amd as ggnn
    from oracle import ggnn_ref as R
    c = _random_case(seed)
    og = R.Graph(c["base"], c["K"], c["L"], s=c["s"], seed=c["seed"])
    b = torch.from_numpy(c["base"]).cuda()
    ggnn.set_cache_mode(mode)
    try:
        g = ggnn.graph_create(b, c["K"], c["L"], seed=c["seed"], segment_size=c["s"])
        for l in range(c["L"]):
            og.edges(l)[:] = c["layers"][l]
            if l >= 1:
                og.to_lower(l)[:] = c["to_lower"][l]
                og.to_base(l)[:] = c["to_base"][l]
            g.import_layer(l, c["layers"][l], c["to_lower"][l], c["to_base"][l])
        og.stats()[:] = c["stats"]
        g.import_dnn(None, *c["stats"])
        q = torch.from_numpy(c["queries"]).cuda()
        for every in (False, True):
            ids, d, cnt = g.query(q, c["k"], c["beam"], c["tau"], pq_cap=c["P"], visited_cap=c["V"], max_iter=c["it"],
                                  every_layer=every, counters=True)
            rids, rd, rcnt = og.query(c["queries"], c["k"], c["beam"], c["tau"], pq_cap=c["P"], visited_cap=c["V"],
                                      max_iter=c["it"], every_layer=every, counters=True)
            info = "seed %d N %d K %d L %d D %d k %d beam %d P %d V %d it %d tau %g every %s" % (
                seed, c["N"], c["K"], c["L"], c["D"], c["k"], c["beam"], c["P"], c["V"], c["it"], c["tau"], every)
            assert np.array_equal(ids.cpu().numpy(), rids), info
            assert np.array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32)), info
            assert np.array_equal(cnt.cpu().numpy().astype(np.uint32)[:, :2], rcnt), info
        # bottom layer alone, from start points of the caller's choice
        rng = np.random.default_rng(seed + 1000)
        starts = rng.choice(c["N"], int(rng.integers(1, min(64, c["N"]) + 1)), replace=False).astype(np.int32)
        ids, d, cnt = g.query(q, c["k"], c["beam"], c["tau"], pq_cap=c["P"], visited_cap=c["V"], max_iter=c["it"],
                              counters=True, start_ids=torch.from_numpy(starts).cuda())
        rids, rd, rcnt = og.query(c["queries"], c["k"], c["beam"], c["tau"], pq_cap=c["P"], visited_cap=c["V"],
                                  max_iter=c["it"], counters=True, start_ids=starts)
        assert np.array_equal(ids.cpu().numpy(), rids), "start points, seed %d" % seed
        assert np.array_equal(d.cpu().numpy().view(np.uint32), rd.view(np.uint32))
        assert np.array_equal(cnt.cpu().numpy().astype(np.uint32)[:, :2], rcnt)
    finally:
        ggnn.set_cache_mode(0)
