"""GPU tests at sizes where 32 bits run out: vector arrays of more than 4 GiB (64-bit row offsets) and
layers or batches of more items than one kernel launch can hold (launches in chunks)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _segment_of(R, seed, N, G0, row):
    """members (base rows) of the bottom segment that holds `row`, from the oracle's partition"""
    pos = R.perm_inv(seed, N, int(row))
    seg = ((pos + 1) * G0 - 1) // N
    lo, hi = seg * N // G0, (seg + 1) * N // G0
    return [R.perm(seed, N, p) for p in range(lo, hi)]


def _check_segment_rows(R, base_t, rows, sample, seed, N, G0, K):
    """rows[z] must hold the K nearest members of z's own segment, ascending by (distance, id)"""
    for z in sample:
        mem = np.array([m for m in _segment_of(R, seed, N, G0, z) if m != z], np.int64)
        x = base_t[torch.from_numpy(mem).cuda()].cpu().numpy().astype(np.int64)
        zq = base_t[int(z)].cpu().numpy().astype(np.int64)
        d2 = ((x - zq) ** 2).sum(1)
        order = mem[np.lexsort((mem, d2))][:K]
        want = np.full(K, -1, np.int64)
        want[:len(order)] = order
        assert np.array_equal(rows[int(z)].astype(np.int64), want), int(z)


def test_vector_array_above_4_gib_sampled_parity():
    """40M x 128 uint8 rows (5.12 GB): byte offsets of the last 6.4M rows do not fit 32 bits, so the kernels
    with 64-bit row offsets run.  (i) After Merge(0, 0) sampled rows -- among them the last rows of the
    array -- hold exactly the nearest members of their own segment (numpy, exact integer distances).
    (ii) After the whole construction, sampled queries equal the oracle's search of the exported graph
    bit for bit, results reach into the part of the array beyond 4 GiB, and every reported distance is the
    exact one."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import ggnn_inputs
    import paper_1912_01059_amd as ggnn
    from oracle import ggnn_ref as R
    ggnn.set_cache_mode(0)
    cfg = ggnn_inputs.CONFIGS["sift100m_u8"]
    dev = torch.device("cuda:0")
    N, K, L, seed = 40_000_000, 24, 4, 42
    b = ggnn_inputs.gmm_int_torch(N, 128, cfg["components"], cfg["sigma"], cfg["data_seed"], cfg["data_seed"] + 1, dev, "u8")
    q = ggnn_inputs.gmm_int_torch(2000, 128, cfg["components"], cfg["sigma"], cfg["data_seed"], cfg["query_seed"], dev, "u8")
    assert b.numel() * b.element_size() > 2 ** 32
    g = ggnn.graph_create(b, K, L, seed=seed, visited_cap=32, max_iter=32, refinements=1)
    G0 = g.g ** (L - 1)
    g.merge(0, 0)
    rows, _, _ = g.export_layer(0)
    rng = np.random.default_rng(1)
    first_far = 2 ** 32 // 128
    sample = np.concatenate([[0, 1, first_far - 1, first_far, first_far + 1, N - 2, N - 1],
                             rng.integers(0, N, 40), rng.integers(first_far, N, 40)])
    _check_segment_rows(R, b, rows, sample, seed, N, G0, K)
    del rows
    g.build_steps()
    k = 10
    ids, dists, cnt = g.query(q, k, 10, 0.08, visited_cap=64, every_layer=True, counters=True)
    ids, dists, cnt = ids.cpu().numpy(), dists.cpu().numpy(), cnt.cpu().numpy()
    assert (ids >= 0).all() and (ids < N).all()
    assert (ids >= first_far).any()
    key = (dists.view(np.uint32).astype(np.uint64) << np.uint64(32)) | ids.astype(np.uint64)
    assert (key[:, 1:] > key[:, :-1]).all()
    queries = q.cpu().numpy()
    sample = np.arange(0, len(queries), 20)
    got_rows = b[torch.from_numpy(ids[sample].reshape(-1).astype(np.int64)).cuda()].cpu().numpy().reshape(len(sample), k, 128)
    d2 = ((got_rows.astype(np.int64) - queries[sample][:, None, :].astype(np.int64)) ** 2).sum(2)
    assert np.array_equal(dists[sample], np.sqrt(d2.astype(np.float32)))
    base = b.cpu().numpy()
    og = R.Graph(base, K, L, seed=seed)
    for l in range(g.L):
        e, tl, tb = g.export_layer(l)
        og.edges(l)[:] = e
        if l >= 1:
            og.to_lower(l)[:] = tl
            og.to_base(l)[:] = tb
        del e
    _, mean, mx = g.export_dnn()
    og.stats()[:] = (mean, mx)
    rids, rd, rcnt = og.query(queries[sample], k, 10, 0.08, visited_cap=64, every_layer=True, counters=True)
    assert np.array_equal(ids[sample], rids)
    assert np.array_equal(dists[sample].view(np.uint32), rd.view(np.uint32))
    assert np.array_equal(cnt[sample][:, :2].astype(np.uint32), rcnt)


def test_layer_of_more_points_than_one_launch_holds():
    """70M x 16 uint8 rows: a launch of one 64-lane workgroup per point would need 4.5 * 10^9 work-items in
    one grid dimension, more than a dispatch can count, so the construction kernels run in chunks of 2^24
    workgroups.  After Merge(0, 0) and the symmetric linking of the bottom layer, rows sampled from every
    chunk -- the first and last rows of each, and the last rows of the array -- are complete and correct."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1912_01059_amd as ggnn
    from oracle import ggnn_ref as R
    ggnn.set_cache_mode(0)
    N, D, K, L, seed = 70_000_000, 16, 8, 4, 7
    gen = torch.Generator(device="cuda")
    gen.manual_seed(123)
    b = torch.randint(0, 256, (N, D), generator=gen, device="cuda", dtype=torch.uint8)
    g = ggnn.graph_create(b, K, L, seed=seed, visited_cap=16, max_iter=16, refinements=0)
    assert N * 64 > 2 ** 32
    G0 = g.g ** (L - 1)
    g.merge(0, 0)
    rows, _, _ = g.export_layer(0)
    chunk = 1 << 24
    edges_of_chunks = [c for f in range(0, N, chunk) for c in (f, f + 1, min(N, f + chunk) - 1)]
    sample = np.concatenate([edges_of_chunks, [N - 2, N - 1], np.random.default_rng(2).integers(0, N, 60)])
    _check_segment_rows(R, b, rows, sample, seed, N, G0, K)
    assert (rows[-100_000:] >= 0).all() and (rows[:: 9973] >= 0).all()  # nothing left unwritten
    before = rows[sample].copy()
    del rows
    g.sym(0)
    rows, _, _ = g.export_layer(0)
    cnt = g.export_inv_count(0)
    assert cnt.max() <= K - K // 2 and cnt[-1_000_000:].sum() > 0
    after = rows[sample]
    assert np.array_equal(after[:, : K // 2], before[:, : K // 2])
    for i, z in enumerate(sample):
        row = after[i][after[i] >= 0]
        assert len(set(row.tolist())) == len(row) and int(z) not in row and row.max() < N
        c = cnt[int(z)]
        assert np.array_equal(after[i][: K - c], before[i][: K - c])


def test_batch_of_more_queries_than_one_launch_holds(sift10k):
    """2^24 + 1000 queries (k = 1) on the 10 000-point configuration: the batch is a 1000-query block
    repeated, so query i must get the answer of query i mod 1000 -- in one launch per chunk, and in the
    two-launch path (upper layers, sort, bottom layer), whose workgroup -> query mapping spans the chunks."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1912_01059_amd as ggnn
    ggnn.set_cache_mode(0)
    base, queries, cfg = sift10k
    b = torch.from_numpy(base).cuda()
    g = ggnn.build(b, cfg["K"], cfg["levels"], seed=42, visited_cap=64, max_iter=64)
    block = torch.from_numpy(queries[:1000]).cuda()
    want_ids, want_d = g.query(block, 1, 10, 0.1, visited_cap=16, every_layer=True)
    reps = (1 << 24) // 1000 + 2
    Q = (1 << 24) + 1000
    big = block.repeat(reps, 1)[:Q].contiguous()
    idx = torch.arange(Q, device="cuda") % 1000
    for split_threshold in (1 << 40, 0):  # one launch per chunk; default (two launches for large batches)
        ggnn.set_split_threshold(split_threshold)
        try:
            ids, d = g.query(big, 1, 10, 0.1, visited_cap=16, every_layer=True)
        finally:
            ggnn.set_split_threshold(0)
        assert torch.equal(ids[:, 0], want_ids[idx, 0])
        assert torch.equal(d[:, 0].view(torch.int32), want_d[idx, 0].view(torch.int32))
        del ids, d
