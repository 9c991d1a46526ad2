"""Hand-worked micro-cases for the oracle's search rule and construction steps (no GPU).

Every expected value below was derived with pencil and paper from the paper's rules -- the stopping
criterion d <= d_best_B + tau * min(d_best_1, d_nn) (Eq. 2) with d_nn the maximum first-neighbour
distance for user queries (Eq. 3) and the mean during construction (Eq. 4), the cache operations of
Alg. 2, the layer change of Alg. 4, the hierarchical construction query of Alg. 3 / Alg. 4 and the
symmetric linking of Alg. 5 / Sec. 4.2.1 -- on tiny graphs whose points lie on a line, and is written
out as a literal; the derivation is given step by step in the comment of each case.  Nothing expected
here is computed by the oracle or by a re-implementation of it.

Notation in the comments: id(d) is a cache entry; thr is the right-hand side of Eq. 2; a proposal is
"known" when it sits in best, prioq or visited.  Coordinates are small dyadic numbers, so every
distance |q - x| below is exact in float32.
"""
import numpy as np
import pytest

from oracle import ggnn_ref as R

FAR = [1000.0 + 10.0 * i for i in range(12)]


def _line_graph(xs, rows0, K, s, L, mean, mx, upper=(), seed=1):
    """Graph over the points xs on a line with hand-set layer-0 rows; upper = [(to_lower, to_base, rows)]
    for layers 1.. (rows None = leave empty)."""
    base = np.array(xs, np.float32).reshape(-1, 1)
    g = R.Graph(base, K, L, s=s, seed=seed)
    e = g.edges(0)
    e[:] = -1
    for i, r in enumerate(rows0):
        e[i, :len(r)] = r
    for l, (tl, tb, rows) in enumerate(upper, start=1):
        g.to_lower(l)[:] = tl
        g.to_base(l)[:] = tb
        if rows is not None:
            el = g.edges(l)
            el[:] = -1
            for i, r in enumerate(rows):
                el[i, :len(r)] = r
    g.stats()[:] = (mean, mx)
    return g, base


def _far_rows(first, n):
    """rows of n far-away points first..first+n-1 that only know each other"""
    return [[first + (i + 1) % n, first + (i + 2) % n] for i in range(n)]


def _query(g, x, k, beam, tau, **kw):
    ids, d, cnt = g.query(np.array([[x]], np.float32), k, beam, tau, counters=True, **kw)
    return ids[0].tolist(), d[0].tolist(), cnt[0].tolist()


# ------------------------------------------------------------------------------ Eq. 2 and Eq. 3

def test_slack_uses_the_smaller_of_best_distance_and_dnn_max():
    """Eq. 2 with B = 1, tau = 0.5, user query (d_nn = maximum = 10, the mean is 1), query at 0.
    Points: A=id0 at 4 (start), P=id1 at -5.5, T=id2 at 3.75, P2=id3 at 7, T2=id4 at 0.5; A-[P,P2], P-[T,A],
    T-[P,A], P2-[T2,A], T2-[P2,A]; second start point id5 far away.
      start: A(4) enters the empty cache; id5 (1000) > thr = 4 + 0.5*min(4,10) = 6: rejected.   evals 2
      pop A: P(5.5) <= 6 enters prioq (not best); P2(7) > 6 rejected.                             evals 4
      pop P (5.5 <= 6): A known; T(3.75) enters: best = T, thr = 3.75 + 0.5*min(3.75,10) = 5.625. evals 5
      pop T: P, A known.  prioq empty.                                                            pops 3
    Result T at 3.75.  With max(...) instead of min(...) thr would be 4 + 5 = 9, P2 would be admitted, and
    after T (thr = 3.75 + 5 = 8.75 >= 7) it would be expanded and lead to T2 (0.5); with the mean (1) instead
    of the maximum thr would be 4.5 and P would be rejected (result A)."""
    xs = [4, -5.5, 3.75, 7, 0.5] + FAR[:7]
    rows = [[1, 3], [2, 0], [1, 0], [4, 0], [3, 0]] + _far_rows(5, 7)
    g, _ = _line_graph(xs, rows, K=2, s=2, L=2, mean=1.0, mx=10.0, upper=[([0, 5], [0, 5], None)])
    assert _query(g, 0.0, 1, 1, 0.5, pq_cap=8, visited_cap=8) == ([2], [3.75], [3, 5])


def test_slack_is_bounded_by_dnn_when_the_best_point_is_far():
    """Eq. 2, the other branch of the minimum: d_best_1 = 8 > d_nn = 2 (maximum; mean 0.25), B = 1, tau = 0.5.
    A=id0 at 8 (start), P=id1 at -8.75, T=id2 at 7.5, P2=id3 at 10, T2=id4 at 0.5; rows as in the case above.
      start: A(8); id5 rejected (thr = 8 + 0.5*min(8,2) = 9).                                     evals 2
      pop A: P(8.75) <= 9 enters prioq; P2(10) > 9 rejected.                                      evals 4
      pop P: T(7.5) enters, thr = 7.5 + 0.5*min(7.5,2) = 8.5.                                     evals 5
      pop T: nothing new.                                                                         pops 3
    Result T at 7.5.  With d_best_1 in place of the minimum thr would be 8 + 4 = 12, P2 would be admitted and
    (thr = 7.5 + 3.75 = 11.25 after T) lead to T2; with the mean thr would be 8.125 and P would be rejected."""
    xs = [8, -8.75, 7.5, 10, 0.5] + FAR[:7]
    rows = [[1, 3], [2, 0], [1, 0], [4, 0], [3, 0]] + _far_rows(5, 7)
    g, _ = _line_graph(xs, rows, K=2, s=2, L=2, mean=0.25, mx=2.0, upper=[([0, 5], [0, 5], None)])
    assert _query(g, 0.0, 1, 1, 0.5, pq_cap=8, visited_cap=8) == ([2], [7.5], [3, 5])


def test_threshold_adds_slack_of_the_first_to_the_distance_of_the_last_best():
    """Eq. 2 with B = 2: thr = d_best_2 + tau * min(d_best_1, d_nn), not d_best_2 + tau * min(d_best_2, ...).
    a=id0 at 2 and b=id1 at -6 are the start points, c=id2 at 8, t=id3 at 0.25; a-[c,b], b-[a,c], c-[t,a],
    t-[c,a]; tau = 0.5, d_nn = 10.
      start: a(2), b(6) fill best; thr = 6 + 0.5*min(2,10) = 7.                                   evals 2
      pop a: b known; c(8) > 7 rejected.                                                          evals 3
      pop b (6 <= 7): a known; c is not in the cache, so it is evaluated again and rejected.      evals 4
    Result [a(2), b(6)], 2 pops.  With the slack taken from d_best_2 thr would be 9, c would be admitted
    and would lead to t."""
    xs = [2, -6, 8, 0.25] + FAR[:8]
    rows = [[2, 1], [0, 2], [3, 0], [2, 0]] + _far_rows(4, 8)
    g, _ = _line_graph(xs, rows, K=2, s=2, L=2, mean=1.0, mx=10.0, upper=[([0, 1], [0, 1], None)])
    assert _query(g, 0.0, 2, 2, 0.5, pq_cap=8, visited_cap=8) == ([0, 1], [2.0, 6.0], [2, 4])


# ------------------------------------------------------------------------------ Alg. 2: limits

def test_iteration_limit_cuts_the_search():
    """Alg. 2 Pop with a limit of three iterations on a chain: id i sits at 12 - i and knows i+1 and i-1;
    start points id0 (12) and id1 (11); B = 1, tau = 0.5, d_nn = 10, query at 0.
      start: best = id1(11), prioq = [1(11), 0(12)].                                              evals 2
      pop 1: id2(10) enters (0 known).   pop 2: id3(9).   pop 3: id4(8).                          evals 5
      the fourth pop is refused by the limit although id4(8) <= thr = 8 + 4 = 12.
    Result id4 at 8 after exactly 3 pops; without the limit the chain would be followed to id11 (1)."""
    xs = [12 - i for i in range(12)]
    rows = [[1, 2]] + [[i + 1, i - 1] for i in range(1, 11)] + [[10, 9]]
    g, _ = _line_graph(xs, rows, K=2, s=2, L=2, mean=1.0, mx=10.0, upper=[([0, 1], [0, 1], None)])
    assert _query(g, 0.0, 1, 1, 0.5, pq_cap=4, visited_cap=3, max_iter=3) == ([4], [8.0], [3, 5])
    # the same chain with room for every iteration ends at the nearest point
    ids, d, cnt = _query(g, 0.0, 1, 1, 0.5, pq_cap=4, visited_cap=16, max_iter=16)
    assert (ids, d) == ([11], [1.0])


def test_full_visited_list_forgets_its_oldest_entry():
    """Alg. 2 Pop appends the popped point to a visited list of bounded size; once the list is full the entry
    that has been there longest makes room (the library never lets this happen: it asks for an iteration limit
    within the capacity; the oracle takes any pair).  The chain of the case above (id i at 12 - i, row [i+1,
    i-1], start points id0 and id1, B = 1, tau = 0.5, d_nn = 10, prioq 4, query at 0), four iterations.
    Capacity 1: visited holds the last popped point only.
      start: best = 1(11), prioq = [1(11), 0(12)], thr = 11 + 5 = 16.                               evals 2
      pop 1, visited [1]: 2(10) enters, 0 is in prioq.  best = 2, prioq = [2, 0], thr = 15.         evals 3
      pop 2, visited [2]: 3(9) enters (thr = 13.5); 1 is in no list any more: evaluated, 11 <= 13.5,
        enters prioq = [3(9), 1(11), 0(12)] and falls off best again.                               evals 5
      pop 3, visited [3]: 4(8) enters (thr = 12); 2(10) evaluated again, enters prioq = [4, 2, 1, 0].  evals 7
      pop 4, visited [4]: 5(7) enters (thr = 10.5), prioq = [5, 2, 1, 0]; 3(9) evaluated again, enters:
        prioq = [5, 3, 2, 1].                                                                       evals 9
    Result id5 at 7 after 4 pops and 9 evaluations (6 with room for every popped point).  A list that stops
    taking entries when it is full would keep 1 for good: the second pop evaluates 3 only, the third and the
    fourth two points each: 8 evaluations."""
    xs = [12 - i for i in range(12)]
    rows = [[1, 2]] + [[i + 1, i - 1] for i in range(1, 11)] + [[10, 9]]
    g, _ = _line_graph(xs, rows, K=2, s=2, L=2, mean=1.0, mx=10.0, upper=[([0, 1], [0, 1], None)])
    assert _query(g, 0.0, 1, 1, 0.5, pq_cap=4, visited_cap=1, max_iter=4) == ([5], [7.0], [4, 9])
    assert _query(g, 0.0, 1, 1, 0.5, pq_cap=4, visited_cap=4, max_iter=4) == ([5], [7.0], [4, 6])


def test_visited_list_is_overwritten_in_order_of_arrival():
    """The same chain with capacity 2, the row of id3 changed to [4, 0] and that of id4 to [5, 1]: the list
    runs [1], [1, 2], then 3 takes the place of 1 (the oldest), then 4 the place of 2.
      start 2 evaluations; pop 1: 2 enters (3), 0 is in prioq; pop 2: 3 enters (4), 1 visited;
      pop 3, visited {3, 2}: 4(8) enters (5), thr = 12, 0(12) is still in prioq;
      pop 4, visited {3, 4}: 5(7) enters (6), thr = 10.5; 1 is neither listed nor visited any more: evaluated
      (7) and rejected (11 > 10.5).
    4 pops, 7 evaluations.  Overwriting the newest entry instead would leave {1, 4}, never overwriting {1, 2}:
    either way 1 is still known at the fourth pop and the count is 6."""
    xs = [12 - i for i in range(12)]
    rows = [[1, 2]] + [[i + 1, i - 1] for i in range(1, 11)] + [[10, 9]]
    rows[3] = [4, 0]
    rows[4] = [5, 1]
    g, _ = _line_graph(xs, rows, K=2, s=2, L=2, mean=1.0, mx=10.0, upper=[([0, 1], [0, 1], None)])
    assert _query(g, 0.0, 1, 1, 0.5, pq_cap=4, visited_cap=2, max_iter=4) == ([5], [7.0], [4, 7])


def test_full_prioq_drops_its_largest_entry():
    """Alg. 2 Push into a prioq of one entry on a sparse graph: a=id0 at 5 and b=id1 at 4 are the start
    points, t=id2 at 1 is known to a only, u=id3 at 6; a-[t,b], b-[u,a], t-[a,b], u-[b,a]; B = 2, tau = 0.5,
    d_nn = 10.
      start: a(5) enters; b(4) enters best = [b, a] and displaces a from the one-entry prioq.     evals 2
      thr = 5 + 0.5*min(4,10) = 7.  The layer change re-seeds prioq with the smallest of best: b.
      pop b: u(6) <= 7 enters the (now empty) prioq, not best; a known.                           evals 3
      pop u (6 <= 7): b, a known.  prioq empty.                                                   pops 2
    a is never expanded, so t is never seen: result [b(4), a(5)]."""
    xs = [5, 4, 1, 6] + FAR[:8]
    rows = [[2, 1], [3, 0], [0, 1], [1, 0]] + _far_rows(4, 8)
    g, _ = _line_graph(xs, rows, K=2, s=2, L=2, mean=1.0, mx=10.0, upper=[([0, 1], [0, 1], None)])
    assert _query(g, 0.0, 2, 2, 0.5, pq_cap=1, visited_cap=8) == ([1, 0], [4.0, 5.0], [2, 3])
    # with room for both start points a is expanded and t is found
    ids, d, _ = _query(g, 0.0, 2, 2, 0.5, pq_cap=2, visited_cap=8)
    assert (ids, d) == ([2, 1], [1.0, 4.0])


# ------------------------------------------------------------------------------ Alg. 4: Transform

def test_layer_change_keeps_unpopped_prioq_entries_and_maps_ids():
    """Alg. 4 / Sec. 4.4 (top layer, then bottom layer) with s = 4 start points whose top-layer ids 0..3 are
    the base rows 7, 4, 9, 2 at 5, 3, 9, 4; B = 1, prioq of 3, tau = 0.5, d_nn = 10, query at 0.
      start, in index order: 0(5) enters; 1(3) <= 5 + 2.5 enters, best = 1(3); 2(9) > thr = 3 + 1.5 = 4.5
      rejected; 3(4) <= 4.5 enters prioq only: prioq = [1(3), 3(4), 0(5)].                        evals 4
      layer change: ids become base rows, prioq = [4(3), 2(4), 7(5)] (best is part of it already).
      pop row 4: its neighbours rows 10 and 11 are far: rejected.                                 evals 6
      pop row 2 (4 <= 4.5) -- an entry that was never in best: row 0 at 0.5 enters, best = 0(0.5),
      thr = 0.75; row 4 known.                                                                    evals 7
      pop row 0: rows 2, 4 known.  The head 7(5) > 0.75: end.                                     pops 3
    Result row 0 at 0.5.  If the layer change re-seeded prioq from best alone, row 2 would never be
    expanded and the result would be row 4 at 3."""
    xs = [0.5, 900, 4, 901, 3, 902, 903, 5, 904, 9, 950, 960]
    rows = [[2, 4], [3, 5], [0, 4], [1, 5], [10, 11], [6, 8], [5, 8], [4, 2], [6, 5], [7, 4], [11, 1], [10, 1]]
    g, _ = _line_graph(xs, rows, K=2, s=4, L=2, mean=1.0, mx=10.0, upper=[([7, 4, 9, 2], [7, 4, 9, 2], None)])
    assert _query(g, 0.0, 1, 1, 0.5, pq_cap=3, visited_cap=8) == ([0], [0.5], [3, 7])
    # a prioq of two entries loses 0(5) already during the start; the outcome is the same
    assert _query(g, 0.0, 1, 1, 0.5, pq_cap=2, visited_cap=8) == ([0], [0.5], [3, 7])


def _three_layer(xs, rows0, l1, rows1, l2, **kw):
    """8 points, s = 2, three layers (8 / 4 / 2 points): l1 = base rows of the four layer-1 points,
    l2 = layer-1 ids of the two top points."""
    return _line_graph(xs, rows0, K=2, s=2, L=3, upper=[(l1, l1, rows1), (l2, [l1[i] for i in l2], None)], **kw)


def test_layer_change_truncates_to_the_prioq_capacity_and_restarts_the_iteration_count():
    """Alg. 4 on three layers, two iterations allowed per layer, B = 2, prioq of 2, tau = 0.5, d_nn = 2
    (so the slack is 0.5 * min(d_best_1, 2) = 1), query at 0.  Base rows: a=0 at 10, b=1 at 12, c=2 at 13,
    t=3 at 1 (known to c only), rows 4..7 at 30, 40, 50, 60.  Layer 1 holds rows [a, b, c, 4] as ids 0..3 with
    rows 0-[1,2], 1-[0,2], 2-[1,0], 3-[2,1]; the top layer holds layer-1 ids [0, 3].  Bottom rows: a-[b,5],
    b-[a,5], c-[t,b], t-[c,a], 4-[5,6], 5-[4,6], 6-[5,7], 7-[6,5].
      start: a(10), row 4 (30) fill best; thr = 31.                                               evals 2
      layer 1: pop a: b(12) enters best = [a, b] and prioq = [b(12), 3(30)], thr = 12 + 1 = 13;
               c(13) <= 13 enters prioq only, which drops 3(30): prioq = [b(12), c(13)].          evals 4
               pop b: a, c known.  The third pop is refused by the limit: c(13) stays in prioq.   pops 2
      layer change: best u prioq = [a(10), b(12), c(13)], cut to the two smallest: c is lost.  Count restarts.
      bottom: pop a: b known, row 5 (40) > 13 rejected.  pop b: a known, row 5 evaluated again.   evals 6
              The limit ends the layer.                                                           pops 4
    Result [a(10), b(12)]; t is not found because c was cut.  Had the iteration count not been reset
    the bottom layer would see no pop at all (2 pops in total)."""
    xs = [10, 12, 13, 1, 30, 40, 50, 60]
    rows0 = [[1, 5], [0, 5], [3, 1], [2, 0], [5, 6], [4, 6], [5, 7], [6, 5]]
    rows1 = [[1, 2], [0, 2], [1, 0], [2, 1]]
    g, _ = _three_layer(xs, rows0, [0, 1, 2, 4], rows1, [0, 3], mean=1.0, mx=2.0)
    got = _query(g, 0.0, 2, 2, 0.5, pq_cap=2, visited_cap=2, max_iter=2, every_layer=True)
    assert got == ([0, 1], [10.0, 12.0], [4, 6])


def test_layer_change_empties_visited():
    """Alg. 4: "allow all points to be visited again".  Three layers, B = 1, prioq of 4, tau = 0.5, d_nn = 2.
    Base rows: a=0 at 10, 1 at 20, 2 at 30, t=3 at 1, e=4 at 11, rows 5..7 far.  Layer-1 ids 0..3 are the rows
    [1, 2, 5, a]; the top layer holds layer-1 ids [3, 0] (rows a and 1).  Layer-1 rows: 3-[0,1], others among
    themselves.  Bottom rows: a-[t,e], t-[a,e], e-[a,t].
      start: a(10) enters; row 1 (20) > 10 + 1 = 11 rejected.                                     evals 2
      layer 1: pop id 3 (= a): ids 0 (20) and 1 (30) rejected; prioq empty.  visited = {3}.       evals 4
      layer change to the bottom layer: best = a(10), visited emptied.
      bottom: pop a: t -- base row 3, the number that sat in visited as a layer-1 id -- is a new point:
              t(1) enters, thr = 1 + 0.5 = 1.5; e(11) rejected.                                   evals 6
              pop t: a known, e evaluated again and rejected.                                     evals 7
    Result t at 1 after 3 pops.  With a stale visited list t would be taken for known."""
    xs = [10, 20, 30, 1, 11, 500, 600, 700]
    rows0 = [[3, 4], [2, 5], [1, 5], [0, 4], [0, 3], [6, 7], [5, 7], [6, 5]]
    rows1 = [[1, 2], [0, 2], [0, 1], [0, 1]]
    g, _ = _three_layer(xs, rows0, [1, 2, 5, 0], rows1, [3, 0], mean=1.0, mx=2.0)
    got = _query(g, 0.0, 1, 1, 0.5, pq_cap=4, visited_cap=8, every_layer=True)
    assert got == ([3], [1.0], [3, 7])


# ------------------------------------------------------------------------------ Alg. 3 Merge through Alg. 4

def _merge_toy(mean, mx):
    """8 points in four bottom segments of two (positions 0-1, 2-3, 4-5, 6-7 of the partition order), on a
    line at 0.5, 1, 2, 3.5 | 4.5, 101, 102, 103.  Layer 1: segment 0 = positions (1, 2), segment 1 =
    positions (5, 6); the top layer holds positions (2, 5).  Rows are a hand-set state."""
    N, seed = 8, 5
    pos2row = [R.perm(seed, N, p) for p in range(N)]
    X = [0.5, 1, 2, 3.5, 4.5, 101, 102, 103]
    xs = [0.0] * N
    for p, r in enumerate(pos2row):
        xs[r] = X[p]
    by_pos = [[1, 4], [0, 2], [1, 3], [2, 1], [5, 6], [4, 6], [5, 7], [6, 5]]
    rows0 = [None] * N
    for p, r in enumerate(pos2row):
        rows0[r] = [pos2row[t] for t in by_pos[p]]
    l1 = [pos2row[1], pos2row[2], pos2row[5], pos2row[6]]
    rows1 = [[1, 2], [0, 3], [3, 1], [2, 0]]
    g, base = _line_graph(xs, rows0, K=2, s=2, L=3, mean=mean, mx=mx, seed=seed,
                          upper=[(l1, l1, rows1), ([1, 2], [l1[1], l1[2]], None)])
    assert g.g == 2 and g.n == [8, 4, 2]
    return g, pos2row


def test_merge_searches_from_the_top_segment_of_the_own_subgraph_with_the_mean_in_the_slack():
    """Alg. 3 Merge(l_top = 1, l_m = 0) for z = position 3 (at 3.5), B = K = 2, tau_b = 0.5, mean d_nn = 0.4
    (maximum 3).  z lies in bottom segment 1, whose sub-graph of height 1 is rooted at layer-1 segment
    1 div g = 0: the start points are positions 1 (at 1) and 2 (at 2), not segment 1's (101, 102).
      start: p1(2.5), p2(1.5): best = [p2(1.5), p1(2.5)], thr = 2.5 + 0.5*min(1.5, 0.4) = 2.7 (Eq. 4).
      bottom: pop p2: p1 known, p3 is z itself.  pop p1 (2.5 <= 2.7): p0 at 0.5 (3.0 > 2.7) rejected.
    Row of z = [p2, p1], d_nn1(z) = 1.5.  With the maximum in the slack thr would be 2.5 + 0.75 = 3.25, p0
    would be admitted and would lead to p4 at 4.5 (distance 1): row [p4, p2]."""
    g, pos2row = _merge_toy(mean=0.4, mx=3.0)
    g.merge(1, 0, R.default_params(tau_build=0.5, pq_cap=4, visited_cap=8, max_iter=8))
    z = pos2row[3]
    assert g.edges(0)[z].tolist() == [pos2row[2], pos2row[1]]
    assert g.dnn1()[z] == 1.5
    # position 6 (at 102) belongs to the other sub-graph: start points 101 and 102 (itself, skipped)
    #   start: p5(1) enters.  bottom: pop p5: p4 (97.5): best not full, admitted; p6 is z.  pop p4: p5 known.
    assert g.edges(0)[pos2row[6]].tolist() == [pos2row[5], pos2row[4]]


def test_merge_from_the_top_layer_descends_through_every_layer():
    """Alg. 3 Merge(l_top = 2, l_m = 0) -- the refinement query of Alg. 6 -- for z = position 3 (at 3.5).
      top: positions 2 (1.5) and 5 (97.5) fill best; thr = 97.5 + 0.2.
      layer 1 (ids 0..3 = positions 1, 2, 5, 6): pop id 1 (p2): id 0 = p1 (2.5) enters, best = [p2, p1],
               thr = 2.5 + 0.5*min(1.5, 0.4) = 2.7; id 3 = p6 (98.5) rejected.
               pop id 0 (p1): ids 1, 2 known.  Head p5 (97.5) > 2.7: end.
      bottom: prioq = [p2(1.5), p1(2.5), p5(97.5)].  pop p2: p1 known, p3 = z.  pop p1: p0 (3.0) rejected.
    Row of z = [p2, p1], d_nn1 = 1.5."""
    g, pos2row = _merge_toy(mean=0.4, mx=3.0)
    g.merge(2, 0, R.default_params(tau_build=0.5, pq_cap=4, visited_cap=8, max_iter=8))
    z = pos2row[3]
    assert g.edges(0)[z].tolist() == [pos2row[2], pos2row[1]]
    assert g.dnn1()[z] == 1.5


def test_merge_on_an_upper_layer_stops_at_that_layer():
    """Merge(l_top = 2, l_m = 1): the rows of layer 1 hold layer-1 ids, found without touching the bottom layer.
    z = layer-1 id 0 (position 1, at 1): top points p2 (1) and p5 (100) fill best, thr = 100 + 0.2;
      layer 1: pop id 1 (p2): id 0 is z, id 3 = p6 (101) > 100.2 rejected.  pop id 2 (p5, 100 <= 100.2): id 3 = p6
      rejected again, id 1 known.  Row of id 0 = [1, 2]."""
    g, pos2row = _merge_toy(mean=0.4, mx=3.0)
    before0 = g.edges(0).copy()
    g.merge(2, 1, R.default_params(tau_build=0.5, pq_cap=4, visited_cap=8, max_iter=8))
    assert g.edges(1)[0].tolist() == [1, 2]
    assert np.array_equal(g.edges(0), before0)


def test_build_runs_the_steps_in_the_order_of_alg3_and_alg6(sift10k):
    """Alg. 3: for every new top layer, select it, then merge and link every layer from it down to the
    bottom; Alg. 6: r times, every layer below the top from the top down.  Replaying that order step by
    step gives the graph the one-call construction gives."""
    base = sift10k[0][:3000]
    p = R.default_params(visited_cap=64, max_iter=64)
    whole = R.Graph(base, 12, 3, seed=3).build(p)
    g = R.Graph(base, 12, 3, seed=3)
    for l_top in range(3):
        if l_top > 0:
            g.select(l_top)
        for l_m in range(l_top, -1, -1):
            g.merge(l_top, l_m, p)
            g.sym(l_m, p)
    for _ in range(2):
        for l_m in (1, 0):
            g.merge(2, l_m, p)
            g.sym(l_m, p)
    for l in range(3):
        assert np.array_equal(g.edges(l), whole.edges(l))


# ------------------------------------------------------------------------------ Alg. 5 / Sec. 4.2.1

def _sym_graph(xs, rows, K):
    g, _ = _line_graph(xs, rows, K=K, s=2, L=2, mean=1.0, mx=2.0, upper=[([0, 1], [0, 1], None)])
    return g


def test_symmetric_linking_searches_the_sphere_around_the_shifted_midpoint():
    """Sec. 4.2.1 with K = 4 (k_nn = 2, k_sym = 2): the search for a path from x back to z is centred on
    q_m = z + 0.4 (x - z) and bounded by |q_m - x| = 0.6 |x - z|.
    Group 1: z=0 at 0, x=1 at 10, y=2 at 1, w=3 at 11; rows z-[y,x], x-[w,y], y-[z,x], w-[x].  Only the pair
      (z, x) needs a search (every other pair has a direct link back): q_m = 4, radius 6, sphere [-2, 10].
      start x(6); pop x: y (3) inside, w (7) outside; pop y: its neighbours contain z: a path exists, no link.
      (With 0.6 in place of 0.4 the sphere would be [2, 10], y outside, and x would receive a link to z.)
    Group 2: z=4 at 200, x=5 at 210, y=6 at 197, w=7 at 211; rows z-[y,x], x-[w,y], y-[z,x], w-[x].  Pair (z, x):
      q_m = 204, radius 6, sphere [198, 210].  start x(6); pop x: w (7) and y (7) are both outside: no path.
      The only candidate is x itself, which has room: x receives the inverse link z in its last free slot.
      (With the radius measured from z -- 10 -- y would be inside and the path over y would be found.)"""
    xs = [0, 10, 1, 11, 200, 210, 197, 211, 500, 501, 600, 601]
    rows = [[2, 1], [3, 2], [0, 1], [1], [6, 5], [7, 6], [4, 5], [5], [9], [8], [11], [10]]
    g = _sym_graph(xs, rows, K=4)
    g.sym(0, R.default_params(tau_build=0.5, pq_cap=8, visited_cap=8, max_iter=8))
    want = np.full((12, 4), -1, np.int32)
    for i, r in enumerate(rows):
        want[i, :len(r)] = r
    want[5] = [7, 6, 4, -1]
    assert np.array_equal(g.edges(0), want)
    assert g.inv_count(0).tolist() == [0, 0, 0, 0, 0, 1, 0, 0, 0, 0, 0, 0]


def test_inverse_link_slots_go_to_the_closest_requests_and_losers_move_on():
    """Alg. 5, last loop, with K = 2 (one true neighbour, one slot for an inverse link per row).
    za=0 at -3 with neighbour xa=1 at 2; zb=2 at 2.25 with neighbour xb=3 at -1.5; xa and xb both have
    p=4 at 0 as neighbour; p's neighbour r=5 at 50 links back to p.  No pair except (p, r) / (r, p) has a
    direct link back, and no search finds a path (r is outside every sphere), so four requests arise, each
    with the points its search admitted, ordered by distance to its own midpoint:
      za: q_m = -1, radius 3:      [p(1),    xa(3)]
      zb: q_m = 0.75, radius 2.25: [p(0.75), xb(2.25)]
      xa: q_m = 1.2, radius 1.2:   [p(1.2)]
      xb: q_m = -0.9, radius 0.9:  [p(0.9)]
    All four ask p first; p has one slot, which goes to the smallest distance: zb.  xb and xa have no other
    candidate: their links are dropped.  za moves on to xa, which has room.
    Result: p-[r, zb], xa-[p, za]; every other row unchanged."""
    xs = [-3, 2, 2.25, -1.5, 0, 50, 500, 501, 600, 601, 700, 701]
    rows = [[1], [4], [3], [4], [5], [4], [7], [6], [9], [8], [11], [10]]
    g = _sym_graph(xs, rows, K=2)
    g.sym(0, R.default_params(tau_build=0.5, pq_cap=8, visited_cap=8, max_iter=8))
    want = np.full((12, 2), -1, np.int32)
    for i, r in enumerate(rows):
        want[i, :len(r)] = r
    want[4] = [5, 2]
    want[1] = [4, 0]
    assert np.array_equal(g.edges(0), want)
    assert g.inv_count(0).tolist() == [0, 1, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0]


def test_path_search_uses_inverse_links_granted_in_earlier_rounds():
    """Alg. 5: the proposals of a visited point are its true neighbours and its inverse links.  K = 4.
    u=0 at 0, v=1 at 4, a=2 at 5, b=3 at 6, s=4 at -0.5; rows u-[v,s], v-[a,b], a-[v,b], b-[a,v], s-[u,v].
    Round 0 (first neighbours): only (u, v) lacks a link back.  q_m = 1.6, radius 2.4: a (3.4) and b (4.4)
      are outside, no path; v has room: v receives the inverse link u.
    Round 1 (second neighbours): only (s, v) lacks a link back.  q_m = 1.3, radius 2.7: start v; pop v: a and
      b outside, but v's inverse link u (1.3) is inside; pop u: its neighbours contain s: path found, no link.
    Result: v-[a, b, u], one inverse link.  A search that ignored inverse links would find no path in
    round 1 and give v a second link, s.
    The far points 5..10 are three mutually linked pairs; id 11 at 800 has the single neighbour id 10 at 701,
    which does not link back: q_m = 760.4, radius 59.4; pop 10: its neighbour 9 (700, at 60.4) is outside:
    no path, 10 has room and receives the inverse link 11 behind its one true neighbour."""
    xs = [0, 4, 5, 6, -0.5, 500, 501, 600, 601, 700, 701, 800]
    rows = [[1, 4], [2, 3], [1, 3], [2, 1], [0, 1], [6], [5], [8], [7], [10], [9], [10]]
    g = _sym_graph(xs, rows, K=4)
    g.sym(0, R.default_params(tau_build=0.5, pq_cap=8, visited_cap=8, max_iter=8))
    want = np.full((12, 4), -1, np.int32)
    for i, r in enumerate(rows):
        want[i, :len(r)] = r
    want[1] = [2, 3, 0, -1]
    want[10] = [9, 11, -1, -1]
    assert np.array_equal(g.edges(0), want)
    assert g.inv_count(0).tolist() == [0, 1, 0, 0, 0, 0, 0, 0, 0, 0, 1, 0]


def _unlinked_pairs(base, rows, inv_count, K, zs):
    """For every pair (z, x), x one of the first K/2 entries of z's row: is z in x's row, or can z be reached
    from x over the rows without leaving the sphere around q_m = z + 0.4 (x - z) that touches x (Sec. 4.2.1)?
    Returns the pairs for which neither holds, with the points of the sphere reachable from x."""
    b64 = base.astype(np.float64)
    knn = K // 2
    direct = path = 0
    rest = []
    for z in zs:
        for x in rows[z, :knn]:
            if x < 0:
                continue
            if z in rows[x]:
                direct += 1
                continue
            qm = b64[z] + 0.4 * (b64[x] - b64[z])
            radius = np.sqrt(((qm - b64[x]) ** 2).sum()) * (1 + 1e-6)
            inside, todo, found = {int(x)}, [int(x)], False
            while todo and not found:
                a = todo.pop()
                for b in rows[a]:
                    if b == z:
                        found = True
                        break
                    if b >= 0 and int(b) not in inside and np.sqrt(((qm - b64[b]) ** 2).sum()) <= radius:
                        inside.add(int(b))
                        todo.append(int(b))
            if found:
                path += 1
            else:
                rest.append((z, int(x), inside))
    return direct, path, rest


def test_unlinked_pairs_have_a_path_inside_the_sphere_or_no_room(sift10k, sift10k_oracle_graph):
    """Sec. 4.2 / Alg. 5: after symmetric linking, for every point z and each of its k_nn nearest neighbours x,
    either x links back to z, or z can be reached from x inside the sphere of Sec. 4.2.1 (breadth-first
    search over the rows, in numpy), or the link had to be dropped for lack of room: every candidate of
    the failed search -- the up to K points closest to q_m that it admitted, x among them whenever the
    sphere holds at most K reachable points -- had all its k_sym slots taken."""
    base, _, cfg = sift10k
    K = cfg["K"]
    ksym = K - K // 2
    # (i) the first linking pass of the construction: segments of about 30 points, linked inside the segment
    g = R.Graph(base, K, cfg["levels"])
    p = R.default_params()
    g.merge(0, 0, p)
    g.sym(0, p)
    rows, cnt = g.edges(0), g.inv_count(0)
    direct, path, rest = _unlinked_pairs(base, rows, cnt, K, range(0, 10_000, 5))
    assert path > 0 and direct > 10 * path
    for z, x, inside in rest:
        assert len(inside) > K or cnt[x] == ksym, (z, x)
        assert any(cnt[a] == ksym for a in inside)
    assert len(rest) < 0.01 * (direct + path)
    # (ii) the finished graph (the first k_nn entries of a row are the merge results the pass started from)
    rows, cnt = sift10k_oracle_graph.edges(0), sift10k_oracle_graph.inv_count(0)
    direct, path, rest = _unlinked_pairs(base, rows, cnt, K, range(0, 10_000, 4))
    for z, x, inside in rest:
        assert len(inside) > K or cnt[x] == ksym, (z, x)
        assert any(cnt[a] == ksym for a in inside)
    assert direct > 2 * len(rest)
