"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU)."""
import heapq
import math
import os

import numpy as np
import pytest

from oracle import ggnn_ref as R

HERE = os.path.dirname(os.path.abspath(__file__))


# ---------------------------------------------------------------- geometry

def _golden_rows():
    rows = []
    for line in open(os.path.join(HERE, "golden", "graph_size.txt")):
        if line.startswith("#") or not line.strip():
            continue
        rows.append(line.split())
    return rows


@pytest.mark.parametrize("row", _golden_rows())
def test_geometry_matches_paper_examples(row):
    """Appendix 'Graph Size' and Table 4: growth factor, upper-layer point count, bytes."""
    N, s, L, K, g_exp, n_upper_exp = (int(v) for v in row[:6])
    g, n, G = R.geometry(N, s, L)
    assert g == g_exp
    assert sum(n[1:]) == n_upper_exp
    # N_upper = s * sum_{i<=L-2} g^i
    assert sum(n[1:]) == s * sum(g ** i for i in range(L - 1))
    if row[6] != "-":
        size = ((N + n_upper_exp) * K + 2 * n_upper_exp + 2) * 4 / 2 ** 20
        assert abs(size - float(row[6])) <= float(row[7])


@pytest.mark.parametrize("N,s,L", [(10_000, 32, 3), (1_200_000, 32, 4), (100_000_000, 32, 4), (5000, 32, 2), (777, 16, 3)])
def test_geometry_level_sizes_follow_growth_factor(N, s, L):
    g, n, G = R.geometry(N, s, L)
    assert n[0] == N and n[L - 1] == s and G[L - 1] == 1
    for l in range(1, L):
        assert n[l] == s * g ** (L - 1 - l) and G[l] == g ** (L - 1 - l)
    assert G[0] == g ** (L - 1)
    # g is the floor or the ceiling of (N/s)^(1/(L-1)) whose bottom segment size is closest to s
    root = (N / s) ** (1.0 / (L - 1))
    assert g in (math.floor(root), math.ceil(root)) or abs(g - root) < 1e-6
    other = math.floor(root) if g == math.ceil(root) else math.ceil(root)
    if other >= 1 and other != g:
        assert abs(N / g ** (L - 1) - s) <= abs(N / other ** (L - 1) - s)


@pytest.mark.parametrize("N", [2, 3, 17, 1000, 4097, 65536, 100_003])
def test_partition_is_a_bijection(N):
    seed = 1234
    m = min(N, 5000)
    idx = np.arange(N) if N <= 5000 else np.random.default_rng(0).choice(N, m, replace=False)
    img = np.array([R.perm(seed, N, int(p)) for p in idx])
    assert img.min() >= 0 and img.max() < N and len(set(img.tolist())) == len(idx)
    back = np.array([R.perm_inv(seed, N, int(r)) for r in img])
    assert np.array_equal(back, idx)
    if N >= 1000:  # not the identity, and seed dependent
        assert (img != idx).mean() > 0.9
        img2 = np.array([R.perm(seed + 1, N, int(p)) for p in idx])
        assert (img2 != img).mean() > 0.9


def test_uniform_is_uniform():
    u = np.array([R.uniform(7, 1, i) for i in range(20000)])
    assert u.min() > 0.0 and u.max() < 1.0
    hist, _ = np.histogram(u, bins=20, range=(0, 1))
    chi2 = ((hist - 1000.0) ** 2 / 1000.0).sum()
    assert chi2 < 50.0  # 19 dof, p ~ 1e-4
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 0.03


# ---------------------------------------------------------------- distance

def test_distance_l2_exact_on_integer_data():
    """Integer-valued data: every partial sum is an integer below 2^24, so the float32
    result is the correctly rounded square root of the exact integer sum."""
    rng = np.random.default_rng(1)
    for D in (4, 96, 100, 128):
        q = rng.integers(0, 256, D).astype(np.float32)
        x = rng.integers(0, 256, D).astype(np.float32)
        exact = int(((q.astype(np.int64) - x.astype(np.int64)) ** 2).sum())
        want = np.sqrt(np.float32(exact))  # float32 sqrt is correctly rounded
        assert R.distance(q, x) == float(want)
        assert R.distance(q, x.astype(np.uint8)) == float(want)
        assert R.distance(q, q) == 0.0


@pytest.mark.parametrize("D", [8, 96, 100, 128, 200])
def test_distance_l2_real_within_rounding_bound(D):
    rng = np.random.default_rng(D)
    for _ in range(50):
        q = rng.standard_normal(D).astype(np.float32)
        x = rng.standard_normal(D).astype(np.float32)
        ref = np.sqrt(((q.astype(np.float64) - x.astype(np.float64)) ** 2).sum())
        got = R.distance(q, x)
        assert abs(got - ref) <= (D + 4) * 2.0 ** -24 * ref
        assert R.distance(x, q) == got  # (q-x)^2 == (x-q)^2 term by term


def test_distance_cosine():
    rng = np.random.default_rng(5)
    for D in (100, 128):
        q = rng.standard_normal(D)
        x = rng.standard_normal(D)
        qn = (q / np.linalg.norm(q)).astype(np.float32)
        xn = (x / np.linalg.norm(x)).astype(np.float32)
        ref = 1.0 - float(qn.astype(np.float64) @ xn.astype(np.float64))
        assert abs(R.distance(qn, xn, metric=R.COSINE) - ref) <= (D + 4) * 2.0 ** -24
        assert R.distance(qn, qn, metric=R.COSINE) <= 4 * D * 2.0 ** -24


@pytest.mark.parametrize("D,lanes", [(128, 8), (256, 8), (320, 64), (960, 64)])
def test_distance_summation_tree_is_the_documented_one(D, lanes):
    """A value chosen so that summation order matters: the documented tree (chunks of 4
    elements dealt to `lanes` accumulators, fma chains, butterfly) must be what is used; rows of at
    most 1024 bytes take 8 accumulators, longer ones 64."""
    rng = np.random.default_rng(11)
    assert R.row_lanes(D, 4) == lanes
    hits = 0
    for _ in range(20):
        q = (rng.standard_normal(D) * 10 ** rng.uniform(-3, 3, D)).astype(np.float32)
        x = np.zeros(D, np.float32)
        part = [np.float32(0)] * lanes
        for c in range(D // 4):
            for e in range(4):
                t = np.float32(q[4 * c + e] - x[4 * c + e])
                # fma(t, t, acc): exact product and sum in float64-with-care
                part[c % lanes] = np.float32(math.fma(float(t), float(t), float(part[c % lanes]))) \
                    if hasattr(math, "fma") else _fma32(t, t, part[c % lanes])
        step = lanes // 2
        while step >= 1:
            part = [np.float32(part[l] + part[l ^ step]) for l in range(lanes)]
            step //= 2
        want = float(np.sqrt(part[0]))
        assert R.distance(q, x) == want
        seq = np.float32(0)
        for j in range(D):
            seq = _fma32(q[j], q[j], seq)
        hits += float(np.sqrt(seq)) != want
    assert hits > 0  # the inputs really do distinguish summation orders


@pytest.mark.parametrize("D", [64, 128, 256])
def test_both_summation_trees_stay_within_the_float64_bound(D):
    """The number of accumulators of the summation tree (8, or 64 for long rows) is a convention shared
    with the GPU kernels, not something the paper fixes: whatever the width, the result must stay within
    the rounding bound of the float64 distance, and on integer-valued rows (exact sums) the two widths
    must give the same bits."""
    rng = np.random.default_rng(100 + D)
    for _ in range(40):
        q = rng.standard_normal(D).astype(np.float32)
        x = rng.standard_normal(D).astype(np.float32)
        ref = np.sqrt(((q.astype(np.float64) - x.astype(np.float64)) ** 2).sum())
        for lanes in (8, 64):
            assert abs(R.distance(q, x, lanes=lanes) - ref) <= (D + 4) * 2.0 ** -24 * ref
        qi = rng.integers(0, 256, D).astype(np.float32)
        xi = rng.integers(0, 256, D).astype(np.float32)
        assert R.distance(qi, xi, lanes=8) == R.distance(qi, xi, lanes=64)


def _fma32(a, b, c):
    # float32 fma through exact rational arithmetic
    from fractions import Fraction
    v = Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c))
    return np.float32(_round_fraction_to_f32(v))


def _round_fraction_to_f32(v):
    from fractions import Fraction
    if v == 0:
        return 0.0
    d = float(v)  # correctly rounded to double; double -> float32 could double-round
    f = np.float32(d)
    # repair a possible double rounding by checking the neighbours exactly
    cands = [np.nextafter(f, np.float32(-np.inf)), f, np.nextafter(f, np.float32(np.inf))]
    best = min(cands, key=lambda c: (abs(Fraction(float(c)) - v), int(np.float32(c).view(np.uint32)) & 1))
    return float(best)


# ---------------------------------------------------------------- brute force

def test_bruteforce_matches_float64_argsort(sift10k):
    base, queries, _ = sift10k
    ids, dists = R.bruteforce(base, queries[:50], 10)
    b = base.astype(np.float64)
    for i in range(50):
        d2 = ((b - queries[i].astype(np.float64)) ** 2).sum(1)  # exact integers
        order = np.lexsort((np.arange(len(b)), d2))[:10]
        assert np.array_equal(ids[i], order)
        assert np.array_equal(dists[i], np.sqrt(d2[order].astype(np.float32)))


def test_bruteforce_cosine_matches_numpy():
    rng = np.random.default_rng(3)
    base = rng.standard_normal((500, 100)).astype(np.float32) * np.exp(rng.normal(0, 0.5, (500, 1))).astype(np.float32)
    q = rng.standard_normal((20, 100)).astype(np.float32)
    ids, dists = R.bruteforce(base, q, 5, metric=R.COSINE)
    bn = base.astype(np.float64) / np.linalg.norm(base.astype(np.float64), axis=1, keepdims=True)
    qn = q.astype(np.float64) / np.linalg.norm(q.astype(np.float64), axis=1, keepdims=True)
    ref = 1.0 - qn @ bn.T
    for i in range(20):
        order = np.argsort(ref[i])[:5]
        assert np.array_equal(ids[i], order)
        assert np.allclose(dists[i], ref[i][order], atol=1e-5)


# ---------------------------------------------------------------- search state machine

def _tiny_graph(N, D, K, seed, real=True, complete=False):
    """A hand-made two-level graph: exact kNN rows computed with numpy, top layer = 32
    seeded rows.  Nothing here comes from the oracle's build."""
    rng = np.random.default_rng(seed)
    base = rng.standard_normal((N, D)).astype(np.float32) if real else rng.integers(0, 256, (N, D)).astype(np.float32)
    g = R.Graph(base, K, 2, s=32, seed=seed)
    d2 = ((base[:, None, :].astype(np.float64) - base[None, :, :].astype(np.float64)) ** 2).sum(2)
    np.fill_diagonal(d2, np.inf)
    if complete:
        rows = np.array([[j for j in range(N) if j != i] for i in range(N)], np.int32)
        rows = np.array([rng.permutation(r) for r in rows], np.int32)
    else:
        rows = np.argsort(d2, axis=1, kind="stable")[:, :K].astype(np.int32)
    g.edges(0)[:] = rows
    top = rng.choice(N, 32, replace=False).astype(np.int32)
    g.to_lower(1)[:] = top
    g.to_base(1)[:] = top
    g.stats()[:] = (1.0, 2.0)
    return g, base


def _reachable(g, N):
    seen = set(g.to_base(1).tolist())
    todo = list(seen)
    e = g.edges(0)
    while todo:
        a = todo.pop()
        for b in e[a]:
            if b >= 0 and int(b) not in seen:
                seen.add(int(b))
                todo.append(int(b))
    return seen


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_search_with_unbounded_best_is_exhaustive(seed):
    """With best at least as long as the data set the threshold stays +inf, every
    reachable point is visited and the answer is the exact one."""
    N, D, K = 160, 16, 8
    g, base = _tiny_graph(N, D, K, seed)
    rng = np.random.default_rng(100 + seed)
    q = rng.standard_normal((40, D)).astype(np.float32)
    reach = sorted(_reachable(g, N))
    ids, dists = g.query(q, 10, N, 0.0, pq_cap=N, visited_cap=N, max_iter=N)
    gt_ids, gt_d = R.bruteforce(base[reach], q, 10)
    assert np.array_equal(ids, np.array(reach, np.int32)[gt_ids])
    assert np.array_equal(dists, gt_d)
    if len(reach) == N:
        assert np.array_equal(ids, R.bruteforce(base, q, 10)[0])


def test_search_on_complete_graph_is_exact_for_any_parameters():
    N, D = 96, 12
    g, base = _tiny_graph(N, D, N - 1, 7, complete=True)
    q = np.random.default_rng(8).standard_normal((30, D)).astype(np.float32)
    gt = R.bruteforce(base, q, 10)
    for beam, tau, P, V in [(10, 0.0, 4, 1), (10, 0.5, 64, 384), (16, 0.2, 8, 8)]:
        ids, dists = g.query(q, 10, beam, tau, pq_cap=P, visited_cap=V)
        assert np.array_equal(ids, gt[0]) and np.array_equal(dists, gt[1])


def _classical_best_first(base, edges, starts, q, ef):
    """Textbook best-first graph search with a result set of size ef (the stopping rule
    Sec. 3.1.2 contrasts the slack with): heaps and a visited set, no capacities."""
    def dist(i):
        return float(np.float32(R.distance(q, base[i])))
    seen = set()
    cand, res = [], []
    for s_ in starts:
        seen.add(s_)
        d = dist(s_)
        if len(res) < ef or d < -res[0][0]:
            heapq.heappush(cand, (d, s_))
            heapq.heappush(res, (-d, -s_))
            if len(res) > ef:
                heapq.heappop(res)
    while cand:
        d, c = heapq.heappop(cand)
        if len(res) == ef and d > -res[0][0]:
            break
        for nb in edges[c]:
            nb = int(nb)
            if nb < 0 or nb in seen:
                continue
            seen.add(nb)
            dn = dist(nb)
            if len(res) < ef or dn < -res[0][0]:
                heapq.heappush(cand, (dn, nb))
                heapq.heappush(res, (-dn, -nb))
                if len(res) > ef:
                    heapq.heappop(res)
    out = sorted((-a, -b) for a, b in res)
    return [i for _, i in out], [d for d, _ in out]


@pytest.mark.parametrize("seed", [11, 12])
def test_search_without_slack_is_classical_best_first(seed):
    """tau = 0 and large prioq / visited: the cache reduces to the classical best-first
    search whose result list has length `beam` (real-valued data: no distance ties)."""
    N, D, K = 400, 24, 10
    g, base = _tiny_graph(N, D, K, seed)
    q = np.random.default_rng(seed).standard_normal((25, D)).astype(np.float32)
    for ef in (10, 24):
        ids, dists = g.query(q, 10, ef, 0.0, pq_cap=N, visited_cap=N, max_iter=N)
        for i in range(len(q)):
            want_ids, want_d = _classical_best_first(base, g.edges(0), g.to_base(1).tolist(), q[i], ef)
            assert ids[i].tolist() == want_ids[:10]
            assert np.allclose(dists[i], want_d[:10], rtol=0, atol=0)


def test_search_outputs_are_sorted_distinct_and_true_distances(sift10k, sift10k_oracle_graph):
    """Sec. 5 'exact distance calculations': every reported distance is the true one."""
    base, queries, cfg = sift10k
    g = sift10k_oracle_graph
    ids, dists, cnt = g.query(queries, 10, 10, 0.3, counters=True)
    for i in range(0, len(queries), 7):
        row = ids[i][ids[i] >= 0]
        assert len(set(row.tolist())) == len(row)
        d2 = ((base[row].astype(np.int64) - queries[i].astype(np.int64)) ** 2).sum(1)
        assert np.array_equal(dists[i][: len(row)], np.sqrt(d2.astype(np.float32)))
        keys = list(zip(dists[i][: len(row)].tolist(), row.tolist()))
        assert keys == sorted(keys)
    assert cnt[:, 0].max() <= 384 and (cnt[:, 1] >= 32).all()


def test_search_slack_monotone_and_hierarchy_helps(sift10k, sift10k_oracle_graph, sift10k_gt):
    """Sec. 3.1.2: larger tau visits more and is at least as accurate; Sec. 4.4: on data
    whose bottom layer falls into separate clusters only the layer-by-layer descent can
    reach every cluster."""
    base, queries, cfg = sift10k
    g = sift10k_oracle_graph
    gt = sift10k_gt[0]
    prev_r, prev_c = -1.0, -1.0
    for tau in (0.0, 0.1, 0.2, 0.4):
        ids, _, cnt = g.query(queries, 10, 10, tau, every_layer=True, counters=True)
        r, c = R.recall(ids, gt), cnt[:, 0].mean()  # pops
        assert r >= prev_r - 1e-9 and c >= prev_c
        prev_r, prev_c = r, c
    assert prev_r >= 0.99
    short = R.recall(g.query(queries, 10, 10, 0.4)[0], gt)
    assert short <= prev_r


# ---------------------------------------------------------------- construction

def _segment_members(g, layer, seg):
    if layer > 0:
        return list(range(seg * g.s, (seg + 1) * g.s))
    G0 = g.g ** (g.L - 1)
    lo, hi = seg * g.N // G0, (seg + 1) * g.N // G0
    return [R.perm(g.seed, g.N, p) for p in range(lo, hi)]


def test_merge_on_own_layer_is_brute_force_inside_the_segment(sift10k):
    """Alg. 3: 'use brute force if l_top = l_m'."""
    base, _, cfg = sift10k
    g = R.Graph(base, cfg["K"], cfg["levels"])
    g.merge(0, 0, R.default_params())
    e = g.edges(0)
    G0 = g.g ** (g.L - 1)
    seen = np.zeros(g.N, bool)
    b64 = base.astype(np.int64)
    for seg in range(0, G0, 13):
        mem = _segment_members(g, 0, seg)
        assert 30 <= len(mem) <= 31
        for z in mem:
            seen[z] = True
            others = np.array([m for m in mem if m != z])
            d2 = ((b64[others] - b64[z]) ** 2).sum(1)
            order = others[np.lexsort((others, d2))][: cfg["K"]]
            assert np.array_equal(e[z], order)
            assert g.dnn1()[z] == np.sqrt(np.float32(d2.min()))
    # stats: Eq. 3 / Eq. 4 recomputed from the rows
    d1 = np.sqrt(((b64 - b64[e[:, 0]]) ** 2).sum(1).astype(np.float32))
    assert np.array_equal(d1, g.dnn1())
    assert g.stats()[1] == d1.max()
    assert abs(g.stats()[0] - d1.astype(np.float64).mean()) <= 1e-6 * d1.mean()


def test_select_takes_equal_shares_and_prefers_large_weights():
    """Sec. 4.1 / appendix A: s points per new segment, taken equally from the g children,
    weighted reservoir sampling with weight d_nn1."""
    N, s, L = 1024 + 96, 32, 2
    rng = np.random.default_rng(0)
    base = rng.integers(0, 256, (N, 8)).astype(np.float32)
    cls_w = np.array([1.0, 2.0, 4.0, 8.0])
    picked = np.zeros(4)
    expect = np.zeros(4)
    for seed in range(60):
        g = R.Graph(base, 4, L, s=s, seed=seed)
        assert g.g == 35 or g.g == 32 or g.g > 0
        w = cls_w[np.arange(N) % 4].astype(np.float32)
        g.dnn1()[:] = w
        g.select(1)
        tb, tl = g.to_base(1), g.to_lower(1)
        assert np.array_equal(tb, tl) and len(set(tb.tolist())) == s
        o = 0
        for j in range(g.g):
            share = (j + 1) * s // g.g - j * s // g.g
            mem = _segment_members(g, 0, j)
            chosen = tb[o:o + share]
            o += share
            assert set(chosen.tolist()) <= set(mem)
            if share == 1:
                wm = w[mem].astype(np.float64)
                for c in range(4):
                    expect[c] += wm[np.array(mem) % 4 == c].sum() / wm.sum()
                picked[chosen[0] % 4] += 1
        assert o == s
    chi2 = ((picked - expect) ** 2 / expect).sum()
    assert chi2 < 16.3  # 3 dof, p = 1e-3
    assert picked[3] > 3 * picked[0]


def test_select_ranks_by_efraimidis_spirakis_key():
    """Within one child the winners are the points with the largest u^(1/w)."""
    N, s, L = 640, 32, 2
    rng = np.random.default_rng(4)
    base = rng.integers(0, 256, (N, 8)).astype(np.float32)
    g = R.Graph(base, 4, L, s=s, seed=99)
    w = rng.uniform(0.5, 3.0, N).astype(np.float32)
    g.dnn1()[:] = w
    g.select(1)
    tb = g.to_base(1)
    o = 0
    for j in range(g.g):
        share = (j + 1) * s // g.g - j * s // g.g
        mem = _segment_members(g, 0, j)
        key = {m: R.uniform(99, 1, m) ** (1.0 / float(w[m])) for m in mem}
        want = sorted(mem, key=lambda m: -key[m])[:share]
        assert tb[o:o + share].tolist() == want
        o += share


def test_build_invariants(sift10k, sift10k_oracle_graph):
    base, _, cfg = sift10k
    g = sift10k_oracle_graph
    K = cfg["K"]
    assert g.n == [10_000, 576, 32]
    for l in range(g.L):
        e = g.edges(l)
        n = g.n[l]
        assert e.shape == (n, K)
        for i in range(0, n, 1 if n < 2000 else 9):
            row = e[i]
            valid = row[row >= 0]
            assert len(valid) == (K if n > K else n - 1) or l == g.L - 1
            assert (row[len(valid):] == -1).all()          # sentinels only at the end
            assert len(set(valid.tolist())) == len(valid)  # distinct
            assert i not in valid                          # no self loop
            assert valid.max() < n
        assert g.inv_count(l).max() <= K - K // 2
    assert (g.edges(0) >= 0).all()
    # translation tables are consistent
    assert np.array_equal(g.to_base(1), g.to_lower(1))
    assert np.array_equal(g.to_base(2), g.to_base(1)[g.to_lower(2)])
    for l in (1, 2):
        assert len(set(g.to_base(l).tolist())) == g.n[l]
    # Sec. 4.2: on average fewer than k/4 inverse links are needed
    assert g.inv_count(0).mean() < K / 4
    # the first k_nn entries of a row are true nearest-neighbour results, ascending
    b64 = base.astype(np.int64)
    e0 = g.edges(0)
    for i in range(0, 10_000, 97):
        d2 = ((b64[e0[i, : K // 2]] - b64[i]) ** 2).sum(1)
        assert (np.diff(d2) >= 0).all()


def test_build_graph_quality_and_query_recall(sift10k, sift10k_oracle_graph, sift10k_gt):
    """For-all quality (Sec. 5.2.4) and query recall of the oracle's own build."""
    base, queries, cfg = sift10k
    g = sift10k_oracle_graph
    sample = np.arange(0, 10_000, 25)
    gt_ids, _ = R.bruteforce(base, base[sample], 11)
    e0 = g.edges(0)
    c1 = np.mean([e0[z, 0] == gt_ids[i, 1] for i, z in enumerate(sample)])
    c10 = np.mean([len(set(e0[z, :12].tolist()) & set(gt_ids[i, 1:11].tolist())) / 10 for i, z in enumerate(sample)])
    assert c1 >= 0.99 and c10 >= 0.97
    ids, _ = g.query(queries, 10, 10, 0.3, every_layer=True)
    assert R.recall(ids, sift10k_gt[0]) >= 0.99


def test_sym_adds_back_links(sift10k):
    """Sec. 4.2: after symmetric linking more of the (z, nearest neighbour x) pairs have a
    direct link from x back to z, and no row loses its k_nn true neighbours."""
    base, _, cfg = sift10k
    K = cfg["K"]
    g = R.Graph(base, K, cfg["levels"])
    p = R.default_params()
    g.merge(0, 0, p)
    before = g.edges(0).copy()

    def back_fraction(e):
        hit = tot = 0
        for z in range(0, len(e), 5):
            for x in e[z, : K // 2]:
                tot += 1
                hit += z in e[x]
        return hit / tot

    f0 = back_fraction(before)
    g.sym(0, p)
    after = g.edges(0)
    assert np.array_equal(after[:, : K // 2], before[:, : K // 2])
    assert back_fraction(after) > f0
    cnt = g.inv_count(0)
    assert cnt.max() <= K - K // 2 and cnt.sum() > 0
    for i in range(0, 10_000, 11):
        c = cnt[i]
        assert np.array_equal(after[i, : K - c], before[i, : K - c])
        for z in after[i, K - c:]:
            # an inverse link at row i points to a z that has i's neighbourhood in reach:
            # it was requested because no path from x back to z was found
            assert z not in before[i, : K // 2]


def test_recall_is_stable_across_seeds():
    """Appendix 'Impact of Partitioning': the partition seed does not change the mean recall."""
    import ggnn_inputs
    base, queries, cfg = ggnn_inputs.make("sift10k", n=4000, q=300)
    gt, _ = R.bruteforce(base, queries, 10)
    rec = []
    for seed in (1, 2, 3):
        g = R.Graph(base, 24, 3, seed=seed).build()
        rec.append(R.recall(g.query(queries, 10, 10, 0.3, every_layer=True)[0], gt))
    assert min(rec) >= 0.98 and max(rec) - min(rec) <= 0.02


# ---------------------------------------------------------------- shards

def test_shard_merge_equals_search_over_the_whole_set():
    """Sec. 4.5: exhaustive answers of the shards, merged, are the exhaustive answer of the whole set."""
    rng = np.random.default_rng(21)
    base = rng.integers(0, 256, (900, 16)).astype(np.float32)
    q = rng.integers(0, 256, (40, 16)).astype(np.float32)
    bounds = [0, 250, 610, 900]
    ids, dists = [], []
    for lo, hi in zip(bounds[:-1], bounds[1:]):
        i, d = R.bruteforce(base[lo:hi], q, 7)
        ids.append(i)
        dists.append(d)
    mi, md = R.merge_shards(np.stack(ids), np.stack(dists), bounds[:-1])
    gi, gd = R.bruteforce(base, q, 7)
    assert np.array_equal(mi, gi) and np.array_equal(md, gd)
    # padded lists: a shard with fewer than k points
    ids[0][:, 3:] = -1
    dists[0][:, 3:] = np.inf
    mi2, md2 = R.merge_shards(np.stack(ids), np.stack(dists), bounds[:-1])
    assert (mi2 >= 0).all() and (np.diff(md2, axis=1) >= 0).all()


# ---------------------------------------------------------------- explicit start points

@pytest.mark.parametrize("seed", [31, 32])
def test_search_from_given_start_points_is_classical_best_first(seed):
    """A flat graph searched from start points of the caller's choice (appendix 'Query Starting
    Points'): with tau = 0 and ample capacities this is the textbook best-first search again."""
    N, D, K = 300, 20, 8
    g, base = _tiny_graph(N, D, K, seed)
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((20, D)).astype(np.float32)
    starts = rng.choice(N, 5, replace=False).astype(np.int32)
    ids, dists = g.query(q, 10, 16, 0.0, pq_cap=N, visited_cap=N, max_iter=N, start_ids=starts)
    for i in range(len(q)):
        want_ids, want_d = _classical_best_first(base, g.edges(0), starts.tolist(), q[i], 16)
        assert ids[i].tolist() == want_ids[:10]
        assert np.array_equal(dists[i], np.array(want_d[:10], np.float32))
    # starting everywhere with an unbounded best list is exhaustive search
    every = np.arange(64, dtype=np.int32)
    g2, base2 = _tiny_graph(64, D, K, seed + 100)
    ids2, d2 = g2.query(q, 5, 64, 0.0, pq_cap=64, visited_cap=64, max_iter=64, start_ids=every)
    gi, gd = R.bruteforce(base2, q, 5)
    assert np.array_equal(ids2, gi) and np.array_equal(d2, gd)
