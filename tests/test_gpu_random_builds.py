"""GPU-vs-oracle construction parity on random shapes and parameter sets: element type and metric,
segment size, levels, out-degree, cache capacities of the construction searches, slack factor,
refinement passes, midpoint constraint on / off.  Every layer's rows, tables, inverse-link counts and
the first-neighbour distances must be identical."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _case(seed):
    from oracle import ggnn_ref as R
    rng = np.random.default_rng(seed)
    while True:
        N = int(rng.integers(150, 2500))
        s = int(rng.choice([8, 16, 32, 64]))
        L = int(rng.choice([2, 3, 4]))
        try:
            _, n, G = R.geometry(N, s, L)
        except ValueError:
            continue
        if -(-N // G[0]) > 64 or n[1] >= N:
            continue
        break
    D = int(rng.choice([4, 8, 16, 32, 64, 96, 128]))
    K = int(rng.integers(2, 41))
    kind = str(rng.choice(["real", "int", "u8", "cosine"]))
    if kind == "u8":
        D = max(16, D - D % 16)
        base = rng.integers(0, 256, (N, D)).astype(np.uint8)
    elif kind == "int":
        base = rng.integers(0, 64, (N, D)).astype(np.float32)  # many distance ties
    else:
        base = rng.standard_normal((N, D)).astype(np.float32)
    V = int(rng.choice([16, 48, 96, 160]))
    return dict(N=N, s=s, L=L, D=D, K=K, kind=kind, base=base, P=int(rng.choice([8, 16, 32, 64])), V=V,
                it=int(rng.integers(V // 2, V + 1)), tau=float(rng.choice([0.1, 0.5, 1.0])), r=int(rng.integers(0, 3)),
                symc=bool(rng.integers(0, 2)))


@pytest.mark.parametrize("seed", range(30))
def test_build_matches_oracle_on_random_shape(seed):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1912_01059_amd as ggnn
    from oracle import ggnn_ref as R
    c = _case(seed)
    info = "seed %d: %s" % (seed, {k: v for k, v in c.items() if k != "base"})
    mo, mg = (R.COSINE, ggnn.COSINE) if c["kind"] == "cosine" else (R.L2, ggnn.L2)
    og = R.Graph(c["base"], c["K"], c["L"], s=c["s"], metric=mo, seed=seed).build(
        R.default_params(tau_build=c["tau"], refinements=c["r"], pq_cap=c["P"], visited_cap=c["V"], max_iter=c["it"],
                         sym_constraint=int(c["symc"])))
    ggnn.set_cache_mode(0)
    g = ggnn.build(torch.from_numpy(c["base"]).cuda(), c["K"], c["L"], seed=seed, metric=mg, segment_size=c["s"],
                   tau_build=c["tau"], refinements=(c["r"] if c["r"] > 0 else -1), pq_cap=c["P"], visited_cap=c["V"],
                   max_iter=c["it"], sym_constraint=c["symc"])
    assert g.n == og.n, info
    for l in range(c["L"]):
        e, tl, tb = g.export_layer(l)
        assert np.array_equal(e, og.edges(l)), info + " layer %d" % l
        assert np.array_equal(g.export_inv_count(l), og.inv_count(l)), info
        if l >= 1:
            assert np.array_equal(tl, og.to_lower(l)) and np.array_equal(tb, og.to_base(l)), info
    d, mean, mx = g.export_dnn()
    assert np.array_equal(d.view(np.uint32), og.dnn1().view(np.uint32)) and mx == og.stats()[1], info
