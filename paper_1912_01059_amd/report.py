"""Reports around the hot path, on the synthetic workloads of ggnn_inputs (needs a GPU):

  quality    for-all kNN quality of the built graph: C@1 / C@10 of the bottom-layer rows against
             exhaustive search on a sample of points, and the build-time split (the paper's
             'For-all Queries' table and construction-time composition)
  refine     query recall / speed after r = 0..3 refinement passes (Alg. 6)
  sym        symmetric-linking constraint on / off (Sec. 4.2.1)
  tau_b      construction slack factor against build time and query speed at fixed recall
  batch      queries per second against the number of queries in a batch

Each report prints JSON lines.  Ground truth comes from an exhaustive search with torch (plumbing,
not part of the library)."""
from __future__ import annotations

import argparse
import json
import time


MAX_BLOCK_ELEMS = 1 << 28  # elements of one distance block: torch's float32 matrix product has returned garbage
#                            in the rows of an output beyond 2 GiB on this GPU (500 x 4 000 000), so blocks stay at 1 GiB


def exhaustive(torch, base, queries, k, cosine=False, chunk=500, check=8):
    """Exact k nearest neighbours by exhaustive search with torch: measurement plumbing, not part of the
    library.  Works block by block over the queries and the base rows (MAX_BLOCK_ELEMS) and checks itself:
    the distance of every reported neighbour is recomputed element by element from the two rows (a block of
    queries that fails this is searched again without a matrix product, with a warning on stderr), and for
    `check` queries spread over the batch the k-th distance is compared with a scan of all base rows that uses
    no matrix product.  Raises RuntimeError if a check still fails at the end.  Returns (ids, distances)."""
    import sys
    qs = queries.float()
    if cosine:
        qs = qs / qs.norm(dim=1, keepdim=True)
    n = base.shape[0]
    base_chunk = max(1, MAX_BLOCK_ELEMS // max(1, min(chunk, qs.shape[0])))
    tol = 2e-4 if cosine else 1e-4

    def rows(lo, hi):
        b = base[lo:hi].float()
        return b / b.norm(dim=1, keepdim=True) if cosine else b

    def merge_topk(best, v, i):
        if best is None:
            return v, i
        v2, sel = torch.topk(torch.cat([best[0], v], 1), k, dim=1, largest=False)
        return v2, torch.gather(torch.cat([best[1], i], 1), 1, sel)

    def search(q, with_product):
        best = None
        step = base_chunk if with_product else max(1, (1 << 26) // max(1, q.shape[0] * q.shape[1]))
        for blo in range(0, n, step):
            b = rows(blo, blo + step)
            if not with_product:  # differences (or products) element by element, summed in float64
                dist = ((1.0 - (q[:, None, :].double() * b[None, :, :].double()).sum(2)).clamp_min(0) if cosine
                        else (q[:, None, :].double() - b[None, :, :].double()).pow(2).sum(2).sqrt()).float()
            elif cosine:
                dist = (1.0 - q @ b.T).clamp_min(0)
            else:
                dist = ((q * q).sum(1)[:, None] + (b * b).sum(1)[None, :] - 2.0 * (q @ b.T)).clamp_min(0).sqrt()
            v, i = torch.topk(dist, min(k, b.shape[0]), dim=1, largest=False)
            best = merge_topk(best, v, i + blo)
        return best

    def recompute(q, ii):  # the reported neighbours' distances from the two rows alone, in float64
        nb = base[ii.reshape(-1)].double().reshape(q.shape[0], ii.shape[1], -1)
        if cosine:
            nb = nb / nb.norm(dim=2, keepdim=True)
            return (1.0 - (nb * q.double()[:, None, :]).sum(2)).clamp_min(0)
        return (nb - q.double()[:, None, :]).pow(2).sum(2).sqrt()

    def wrong(q, v, ii):
        again = recompute(q, ii)
        return bool(((again - v.double()).abs() > tol * (1.0 + again)).any())

    ids, d = [], []
    for lo in range(0, qs.shape[0], chunk):
        q = qs[lo:lo + chunk]
        v, ii = search(q, True)
        if wrong(q, v, ii):
            print("exhaustive search: the matrix product gave wrong distances for queries %d..%d; searching them "
                  "again without it" % (lo, lo + q.shape[0] - 1), file=sys.stderr, flush=True)
            v, ii = search(q, False)
            if wrong(q, v, ii):
                raise RuntimeError("exhaustive search: reported distances of queries %d..%d differ from their "
                                   "recomputation" % (lo, lo + q.shape[0] - 1))
        ids.append(ii)
        d.append(v)
    ids, d = torch.cat(ids), torch.cat(d)

    # the k-th distance of a few queries against a scan without a matrix product
    for r in sorted({int(x) for x in torch.linspace(0, qs.shape[0] - 1, min(check, qs.shape[0])).tolist()}):
        q = qs[r].double()
        kth = []
        for blo in range(0, n, 1_000_000):
            b = rows(blo, blo + 1_000_000).double()
            dd = (1.0 - (b * q[None, :]).sum(1)).clamp_min(0) if cosine else (b - q[None, :]).pow(2).sum(1).sqrt()
            kth.append(torch.topk(dd, min(k, dd.shape[0]), largest=False).values)
        want = torch.topk(torch.cat(kth), k, largest=False).values[k - 1]
        if abs(float(want) - float(d[r, k - 1])) > tol * (1.0 + float(want)):
            raise RuntimeError("exhaustive search: query %d, k-th distance %r against %r from the plain scan"
                               % (r, float(d[r, k - 1]), float(want)))
    return ids, d


def recall(dists, gt_d, rel=2e-5):
    k = gt_d.shape[1]
    tol = gt_d[:, k - 1:k] * (1.0 + rel) + 1e-7
    return float(((dists <= tol).sum(1).clamp(max=k).float().mean() / k).item())


def timed_query(torch, g, q, k, beam, slack, limit, every_layer, reps=3):
    ids, d, cnt = g.query(q, k, beam, slack, visited_cap=limit, max_iter=limit, every_layer=every_layer, counters=True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.query(q, k, beam, slack, visited_cap=limit, max_iter=limit, every_layer=every_layer, out=(ids, d), asynchronous=True)
    e1.record()
    torch.cuda.synchronize()
    return d, cnt, e0.elapsed_time(e1) / reps


def graph_quality(torch, g, base, cosine, step):
    sample = torch.arange(0, base.shape[0], step, device=base.device)
    gt, _ = exhaustive(torch, base, base[sample], 11, cosine)
    rows = torch.from_numpy(g.export_layer(0)[0]).to(base.device)[sample]
    knn = g.K // 2
    c1 = (rows[:, 0] == gt[:, 1]).float().mean().item()
    hit = (rows[:, :knn, None] == gt[:, None, 1:11]).any(2).sum(1).float()
    return {"sample": int(sample.numel()), "C@1": round(c1, 4), "C@10": round(float((hit.clamp(max=10) / 10).mean()), 4)}


def main():
    import torch

    import ggnn_inputs
    import paper_1912_01059_amd as ggnn

    ap = argparse.ArgumentParser()
    ap.add_argument("report", choices=["quality", "refine", "sym", "tau_b", "batch"])
    ap.add_argument("--workload", default="sift1m")
    ap.add_argument("--n", type=int, default=None)
    ap.add_argument("--levels", type=int, default=3)
    ap.add_argument("--build-iter", type=int, default=192)
    ap.add_argument("--slack", type=float, default=0.048)
    ap.add_argument("--beam", type=int, default=10)
    ap.add_argument("--limit", type=int, default=48)
    ap.add_argument("--direct", action="store_true", help="drop from the top layer straight to the bottom one")
    a = ap.parse_args()

    base_np, queries_np, cfg = ggnn_inputs.make(a.workload, n=a.n)
    dev = torch.device("cuda:0")
    base, q = torch.from_numpy(base_np).to(dev), torch.from_numpy(queries_np).to(dev)
    cosine = cfg["metric"] == "cosine"
    metric = ggnn.COSINE if cosine else ggnn.L2
    k, K = cfg["k"], cfg["K"]
    _, gt_d = exhaustive(torch, base, q, k, cosine)
    every = not a.direct

    def build(**kw):
        args = dict(seed=42, metric=metric, visited_cap=a.build_iter, max_iter=a.build_iter)
        args.update(kw)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g = ggnn.build(base, K, a.levels, **args)
        torch.cuda.synchronize()
        return g, time.perf_counter() - t0

    def query_line(g):
        d, cnt, ms = timed_query(torch, g, q, k, a.beam, a.slack, a.limit, every)
        c = cnt.double().mean(0).tolist()
        return {"recall": round(recall(d, gt_d), 4), "qps": round(q.shape[0] / ms * 1e3), "pops": round(c[0], 1),
                "rows_gathered": round(c[2], 1)}

    if a.report == "quality":
        g, secs = build()
        out = {"report": "quality", "workload": a.workload, "levels": a.levels, "build_seconds": round(secs, 3),
               "phases_ms": {kk: round(v, 2) for kk, v in g.times().items() if kk.endswith("_ms")}}
        t = g.times()
        tot = t["merge_ms"] + t["sym_ms"] + t["select_ms"] + t["stats_ms"]
        out["split_percent"] = {kk[:-3]: round(100.0 * t[kk] / tot, 2) for kk in ("merge_ms", "sym_ms", "select_ms", "stats_ms")}
        out["graph"] = graph_quality(torch, g, base, cosine, max(1, base.shape[0] // 2000))
        out["inverse_links_per_row"] = round(float(g.export_inv_count(0).mean()), 3)
        out["query"] = query_line(g)
        print(json.dumps(out))
    elif a.report == "refine":
        for r in (0, 1, 2, 3):
            g, secs = build(refinements=r)
            print(json.dumps(dict(report="refine", refinements=r, build_seconds=round(secs, 3),
                                  graph=graph_quality(torch, g, base, cosine, max(1, base.shape[0] // 2000)), **query_line(g))))
            del g
    elif a.report == "sym":
        for on in (True, False):
            g, secs = build(sym_constraint=on)
            print(json.dumps(dict(report="sym", constraint=on, build_seconds=round(secs, 3),
                                  inverse_links_per_row=round(float(g.export_inv_count(0).mean()), 3),
                                  phases_ms={kk: round(v, 2) for kk, v in g.times().items() if kk.endswith("_ms")}, **query_line(g))))
            del g
    elif a.report == "tau_b":
        for tb in (0.1, 0.2, 0.3, 0.5, 0.8):
            g, secs = build(tau_build=tb)
            print(json.dumps(dict(report="tau_b", tau_build=tb, build_seconds=round(secs, 3),
                                  graph=graph_quality(torch, g, base, cosine, max(1, base.shape[0] // 2000)), **query_line(g))))
            del g
    elif a.report == "batch":
        g, secs = build()
        reps = -(-200_000 // q.shape[0])
        big = q.repeat(reps, 1)[torch.randperm(q.shape[0] * reps, device=dev)].contiguous()
        for n in (100, 300, 1000, 3000, 10_000, 30_000, 100_000, 200_000):
            d, cnt, ms = timed_query(torch, g, big[:n].contiguous(), k, a.beam, a.slack, a.limit, every)
            print(json.dumps(dict(report="batch", queries=n, kernel_ms=round(ms, 4), qps=round(n / ms * 1e3))))


if __name__ == "__main__":
    main()
