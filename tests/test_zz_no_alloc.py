"""ggnn_query_static (the entry point that allocates nothing) against ggnn_query_ex, through the C ABI."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_static_workspace_query_matches_query_ex_twice_in_a_row(sift10k):
    """Two calls in a row on one GPU, the second on a smaller batch with other parameters: ids,
    distances and counters are those of ggnn_query_ex(every_layer = 1) bit for bit, whatever the
    static workspace held before.  Sizes beyond the workspace are refused before anything is launched."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1912_01059_amd as ggnn
    base, queries, cfg = sift10k
    b = torch.from_numpy(base).cuda()
    g = ggnn.build(b, cfg["K"], cfg["levels"], seed=42, visited_cap=96, max_iter=96)
    rng = np.random.default_rng(17)
    # (Q, k, beam, slack, prioq): the second call is smaller and must not see the first one's leftovers
    for Q, k, beam, tau, P in [(4000, 10, 10, 0.3, 64), (777, 10, 100, 0.2, 64), (5, 1, 1, 0.0, 32)]:
        q = torch.from_numpy(queries[rng.integers(0, len(queries), Q)].copy()).cuda()
        want_ids, want_d, want_c = g.query(q, k, beam, tau, pq_cap=P, every_layer=True, counters=True)
        ids = torch.full((Q, k), -7, dtype=torch.int32, device="cuda")
        d = torch.full((Q, k), -1.0, dtype=torch.float32, device="cuda")
        c = torch.full((Q, 4), -7, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        ggnn.query_static(g, q, k, beam, tau, (ids, d), pq_cap=P, counters=c)
        assert torch.equal(ids, want_ids)
        assert torch.equal(d.view(torch.int32), want_d.view(torch.int32))
        assert torch.equal(c, want_c)
    # what the workspace cannot hold, or the two-launch search cannot run, is refused with an error
    big = torch.empty((200_000, base.shape[1]), dtype=torch.float32, device="cuda")
    with pytest.raises(ggnn.GgnnError, match="static workspace"):
        ggnn.query_static(g, big, 10, 10, 0.3, (torch.empty((200_000, 10), dtype=torch.int32, device="cuda"),
                                                 torch.empty((200_000, 10), dtype=torch.float32, device="cuda")))
    with pytest.raises(ggnn.GgnnError, match="registers"):
        ggnn.query_static(g, q, 10, 10, 0.3, (torch.empty((len(q), 10), dtype=torch.int32, device="cuda"),
                                              torch.empty((len(q), 10), dtype=torch.float32, device="cuda")), pq_cap=100)
