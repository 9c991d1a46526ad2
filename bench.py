#!/usr/bin/env python3
"""Benchmark of the GGNN hot path on one MI355X.

Workload: the 1M x 128 configuration (float32 integer-valued vectors in [0,255] from a seeded
1024-component Gaussian mixture, 10 000 queries of the same distribution, L2, K=24, k=10).
The graph is built once on the GPU (build seconds are reported); a "step" is one search of the
whole query batch at the operating point that first reaches Recall@10 >= 0.95.  Prints one
JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def ground_truth(torch, base, queries, k, cosine=False, chunk=500):
    """Exact k nearest neighbours by exhaustive search with torch (measurement plumbing, outside
    the timed region).  On integer-valued data every float32 partial sum is an exact integer."""
    b, qs = base.float(), queries.float()
    if cosine:
        b = b / b.norm(dim=1, keepdim=True)
        qs = qs / qs.norm(dim=1, keepdim=True)
    bn = (b * b).sum(1)
    ids, d = [], []
    for lo in range(0, qs.shape[0], chunk):
        q = qs[lo:lo + chunk]
        if cosine:
            dist = (1.0 - q @ b.T).clamp_min(0)
        else:
            dist = ((q * q).sum(1)[:, None] + bn[None, :] - 2.0 * (q @ b.T)).clamp_min(0).sqrt()
        v, i = torch.topk(dist, k, dim=1, largest=False)
        ids.append(i)
        d.append(v)
    return torch.cat(ids), torch.cat(d)


def recall_at_k(dists, gt_d, rel=0.0):
    """Recall@k (the paper's consensus C@k), tolerant of exact distance ties at the k-th place:
    a returned point counts if it is no farther than the k-th true neighbour (times 1 + rel for
    real-valued data, where the exhaustive search's float32 rounding differs from the library's)."""
    k = gt_d.shape[1]
    return float(((dists <= gt_d[:, k - 1:k] * (1.0 + rel)).sum(1).clamp(max=k).float().mean() / k).item())


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="sift1m")
    ap.add_argument("--n", type=int, default=None, help="override the number of base points (debugging)")
    ap.add_argument("--levels", type=int, default=3)
    ap.add_argument("--slack", type=float, default=0.048, help="tau_q of the timed operating point")
    ap.add_argument("--beam", type=int, default=10)
    ap.add_argument("--visited-cap", type=int, default=48, help="visited capacity = iteration limit per layer")
    ap.add_argument("--pq-cap", type=int, default=64)
    ap.add_argument("--large-batch", type=int, default=100_000, help="also time a batch of this many queries (0 = skip)")
    ap.add_argument("--build-iter", type=int, default=192,
                    help="visited capacity = iteration limit per layer of the construction searches")
    ap.add_argument("--sweep", action="store_true", help="also trace the QPS-vs-recall curve")
    ap.add_argument("--direct-drop", action="store_true",
                    help="search the top layer and then the bottom layer only (Sec. 4.4) instead of every layer (Alg. 4)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (reference for hardware byte counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=10_000, help="queries of the oracle's timed search")
    ap.add_argument("--cpu-exhaustive", type=int, default=128, help="queries of the oracle's timed exhaustive search (0 = skip)")
    ap.add_argument("--cpu-build-n", type=int, default=100_000,
                    help="points of the oracle's timed construction (0 = skip; above 10 000: a subset of the workload)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the method shards by replicating the graph "
              "or by independent per-shard graphs); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import ggnn_inputs
    import paper_1912_01059_amd as ggnn

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    base_np, queries_np, cfg = ggnn_inputs.make(args.workload, n=args.n)
    base = torch.from_numpy(base_np).to(dev)
    queries = torch.from_numpy(queries_np).to(dev)
    N, D = base.shape
    Q, k, K = queries.shape[0], cfg["k"], cfg["K"]
    esize = base.element_size()
    metric = ggnn.COSINE if cfg["metric"] == "cosine" else ggnn.L2

    # ---- construction (timed once; the graph stays resident) ----
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    graph = ggnn.build(base, K, args.levels, seed=42, metric=metric, visited_cap=args.build_iter, max_iter=args.build_iter)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    phases = graph.times()

    # roofline of the construction's dominant kernel (merge_kernel): adjacency rows and base rows
    # its searches read, plus the query row and the K results of every search, over the merge time
    n_search = sum(graph.n[l] for l in range(graph.L))  # lower bound on the searches launched
    merge_bytes = phases["merge_pops"] * K * 4 + phases["merge_rows"] * (4 + D * esize)
    build_roofline = {"kernel": "merge_kernel", "bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                      "achieved": round(merge_bytes / (phases["merge_ms"] * 1e-3) / 1e9, 1),
                      "frac": round(merge_bytes / (phases["merge_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                      "pops": int(phases["merge_pops"]), "rows_gathered": int(phases["merge_rows"]),
                      "note": "algorithmic bytes: rows served by the L2 count too, so the rate can exceed the HBM "
                              "peak; HBM-side rates measured with counters are in profiles/"}

    gt_ids, gt_d = ground_truth(torch, base, queries, k, cosine=(metric == ggnn.COSINE))
    rel = 0.0 if cfg["kind"] == "gmm" else 2e-5  # integer-valued rows have exact float32 distances

    # ---- operating point (found with --sweep; the default is the cheapest one that reaches
    # Recall@10 >= 0.95 on this workload) and, on request, the QPS-vs-recall curve ----
    ids = torch.empty((Q, k), dtype=torch.int32, device=dev)
    dists = torch.empty((Q, k), dtype=torch.float32, device=dev)
    chosen = dict(beam=args.beam, slack=args.slack, visited_cap=args.visited_cap, pq_cap=args.pq_cap)
    every = not args.direct_drop
    kw = dict(pq_cap=chosen["pq_cap"], visited_cap=chosen["visited_cap"], every_layer=every)
    curve = []
    if args.sweep:
        sweep = [dict(beam=10, slack=sl, visited_cap=v, pq_cap=64)
                 for (sl, v) in [(0.02, 40), (0.03, 40), (0.04, 48), (0.044, 48), (0.048, 48), (0.05, 56), (0.05, 64),
                                 (0.065, 96), (0.08, 128), (0.1, 192), (0.15, 384), (0.2, 512), (0.3, 1024)]]
        for op in sweep:
            okw = dict(pq_cap=op["pq_cap"], visited_cap=op["visited_cap"], every_layer=every)
            _, _, c = graph.query(queries, k, op["beam"], op["slack"], counters=True, out=(ids, dists), **okw)
            rec = recall_at_k(dists, gt_d, rel)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(3):
                graph.query(queries, k, op["beam"], op["slack"], out=(ids, dists), asynchronous=True, **okw)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 3
            cm = c.double().mean(0).tolist()
            curve.append(dict(op, recall=round(rec, 4), qps=round(Q / ms * 1e3), pops=round(cm[0], 1),
                              dist_evals=round(cm[1], 1)))
    _, _, cnt = graph.query(queries, k, chosen["beam"], chosen["slack"], counters=True, out=(ids, dists), **kw)
    chosen["cnt"] = cnt

    # ---- timed region: exactly `steps` searches of the whole batch ----
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        graph.query(queries, k, chosen["beam"], chosen["slack"], out=(ids, dists), asynchronous=True, **kw)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        graph.query(queries, k, chosen["beam"], chosen["slack"], out=(ids, dists), asynchronous=True, **kw)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    kernel_ms = e0.elapsed_time(e1) / args.steps
    ms_per_step = wall_ms / args.steps
    qps = Q / ms_per_step * 1e3
    final_recall = recall_at_k(dists, gt_d, rel)

    # ---- steady state: a batch large enough to keep every CU busy (the paper's own batch-size
    # study peaks near 95 000 queries), and the rate at which this GPU serves random row gathers
    large = None
    if args.large_batch > 0 and cfg["kind"] == "gmm":
        qn = ggnn_inputs.gmm_int(args.large_batch, D, cfg["components"], cfg["sigma"], cfg["data_seed"],
                                 cfg["query_seed"] + 7, cfg["dtype"])
        ql = torch.from_numpy(qn).to(dev)
        lids, ld, lcnt = graph.query(ql, k, chosen["beam"], chosen["slack"], counters=True, **kw)
        e0l, e1l = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0l.record(stream)
        for _ in range(3):
            graph.query(ql, k, chosen["beam"], chosen["slack"], out=(lids, ld), asynchronous=True, **kw)
        e1l.record(stream)
        torch.cuda.synchronize()
        lms = e0l.elapsed_time(e1l) / 3
        lc = lcnt.double().sum(0).tolist()
        lbytes = len(qn) * (D * esize + k * 8) + lc[0] * K * 4 + lc[2] * (4 + D * esize)
        large = {"queries": len(qn), "qps": round(len(qn) / lms * 1e3, 1), "kernel_ms": round(lms, 3),
                 "achieved_GBps": round(lbytes / (lms * 1e-3) / 1e9, 1),
                 "frac_of_hbm_peak": round(lbytes / (lms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                 "note": "two launches with the bottom-layer searches ordered by region (one part per XCD); algorithmic "
                         "bytes: a good part of the gathered rows is served by the L2"}
        del ql, lids, ld, lcnt
    gather_ceiling = None
    if D * esize <= 512 and metric == ggnn.L2:  # the probe reads rows of up to 512 bytes of the array as given
        n_probe = 12_000_000
        pids = torch.randint(0, N, (n_probe,), device=dev, dtype=torch.int32)
        pout = ggnn.gather_probe(base, pids, 1200)
        torch.cuda.synchronize()
        e0g, e1g = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0g.record(stream)
        for _ in range(3):
            ggnn.gather_probe(base, pids, 1200, out=pout)
        e1g.record(stream)
        torch.cuda.synchronize()
        gather_ceiling = round(n_probe * (D * esize + 4) / (e0g.elapsed_time(e1g) / 3 * 1e-3) / 1e9, 1)
        del pids, pout

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- roofline of the search kernel: algorithmic bytes per launch / kernel time ----
    # per query: the query vector, one adjacency row per pop, one base row (and its id) per row
    # actually gathered (start points included), the k results (ids + distances)
    cnt = chosen["cnt"].double().sum(0).tolist()
    s = graph.s
    algo_bytes = Q * (D * esize + k * 8) + cnt[0] * K * 4 + cnt[2] * (4 + D * esize)
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    # HBM bytes per launch measured with rocprofv3 counters (see profiles/): only valid for the
    # operating point they were taken at
    traffic = None
    op_tag = "operating_point: %s levels=%d beam=%d slack=%g visited_cap=%d pq_cap=%d Q=%d" % (
        args.workload, args.levels, chosen["beam"], chosen["slack"], chosen["visited_cap"], chosen["pq_cap"], Q)
    pmc_path = os.path.join(ROOT, "profiles", "query_kernel_%s_pmc.txt" % args.workload)
    if os.path.exists(pmc_path):
        text = open(pmc_path).read()
        if op_tag in text:
            for line in text.splitlines():
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = int(line.split(":")[1])
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "kernel": "query_kernel",
                "kernel_ms": round(kernel_ms, 3), "algorithmic_bytes_per_launch": int(algo_bytes)}

    # ---- CPU baseline: the oracle's search of the same graph on a sample of the queries ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ggnn_ref as R
        og = R.Graph(base_np, K, args.levels, seed=42, metric=R.COSINE if metric == ggnn.COSINE else R.L2)
        for l in range(graph.L):
            e, tl, tb = graph.export_layer(l)
            og.edges(l)[:] = e
            if l >= 1:
                og.to_lower(l)[:] = tl
                og.to_base(l)[:] = tb
        _, mean, mx = graph.export_dnn()
        og.stats()[:] = (mean, mx)
        ns = min(args.cpu_sample, Q)
        t0 = time.perf_counter()
        rids, rd = og.query(queries_np[:ns], k, chosen["beam"], chosen["slack"], pq_cap=chosen["pq_cap"],
                            visited_cap=chosen["visited_cap"], every_layer=every)
        cpu_s = time.perf_counter() - t0
        same = bool(np.array_equal(rids, ids[:ns].cpu().numpy()) and np.array_equal(rd, dists[:ns].cpu().numpy()))
        # the exhaustive search used for the recall figure, checked against the oracle's on a few queries
        _, bf_d = R.bruteforce(base_np, queries_np[:16], k, metric=R.COSINE if metric == ggnn.COSINE else R.L2)
        gt_ok = bool(np.allclose(bf_d, gt_d[:16].cpu().numpy(), rtol=2e-5, atol=1e-6))
        cores = R.lib().ggnn_ref_num_threads()
        cpu = {"value": round(ns / cpu_s, 1), "unit": "queries/s", "cores": cores,
               "kind": "oracle", "sample": "first %d of the %d queries, same graph and operating point" % (ns, Q),
               "identical_to_gpu": same, "ground_truth_matches_oracle_exhaustive_search": gt_ok}
        # context figures (the paper's CPU references ran on one thread): the same search on one thread,
        # the oracle's exhaustive search, and the oracle's construction of the small configuration
        n1 = min(2000, ns)
        R.lib().ggnn_ref_set_num_threads(1)
        t0 = time.perf_counter()
        og.query(queries_np[:n1], k, chosen["beam"], chosen["slack"], pq_cap=chosen["pq_cap"],
                 visited_cap=chosen["visited_cap"], every_layer=every)
        cpu["single_thread"] = {"value": round(n1 / (time.perf_counter() - t0), 1), "unit": "queries/s", "cores": 1,
                                "sample": "first %d queries" % n1}
        R.lib().ggnn_ref_set_num_threads(cores)
        nb = min(args.cpu_exhaustive, Q)
        if nb > 0:
            t0 = time.perf_counter()
            R.bruteforce(base_np, queries_np[:nb], k, metric=R.COSINE if metric == ggnn.COSINE else R.L2)
            cpu["exhaustive_search"] = {"value": round(nb / (time.perf_counter() - t0), 2), "unit": "queries/s",
                                        "cores": cores, "sample": "first %d queries against all %d points" % (nb, N)}
        if args.cpu_build_n > 0:
            small_np, _, scfg = ggnn_inputs.make(args.workload if args.cpu_build_n > 10_000 else "sift10k",
                                                 n=args.cpu_build_n, q=1)
            sg = R.Graph(small_np, scfg["K"], 3, seed=42)
            t0 = time.perf_counter()
            sg.build(R.default_params(visited_cap=args.build_iter, max_iter=args.build_iter))
            ob_s = time.perf_counter() - t0
            sb = torch.from_numpy(small_np).to(dev)
            ggnn.build(sb, scfg["K"], 3, seed=42, visited_cap=args.build_iter, max_iter=args.build_iter)  # warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            gg = ggnn.build(sb, scfg["K"], 3, seed=42, visited_cap=args.build_iter, max_iter=args.build_iter)
            torch.cuda.synchronize()
            gb_s = time.perf_counter() - t0
            same_graph = all(np.array_equal(gg.export_layer(l)[0], sg.edges(l)) for l in range(3))
            cpu["build"] = {"seconds": round(ob_s, 2), "cores": cores, "gpu_seconds": round(gb_s, 4),
                            "graph_identical_to_gpu": bool(same_graph),
                            "sample": "%d x %d points, K=%d, 3 levels, construction limit %d" % (
                                small_np.shape[0], small_np.shape[1], scfg["K"], args.build_iter)}

    out = {
        "metric": "queries/s at Recall@10>=0.95 (1M x 128 L2, k=10)", "value": round(qps, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if esize == 4 else "u8",
        "data": "synthetic",
        "config": {"workload": "%s: N=%d D=%d Q=%d K=%d k=%d levels=%d" % (args.workload, N, D, Q, K, k, args.levels),
                   "beam": chosen["beam"], "slack": chosen["slack"], "pq_cap": chosen["pq_cap"],
                   "visited_cap": chosen["visited_cap"], "descent": "every layer (Alg. 4)" if every else "top layer, then bottom layer (Sec. 4.4)"},
        "recall_at_10": round(final_recall, 4),
        "build_seconds": round(build_s, 3),
        "build_config": {"levels": args.levels, "K": K, "segment_size": graph.s, "tau_build": 0.5, "refinements": 2,
                         "pq_cap": 64, "visited_cap": args.build_iter, "max_iter": args.build_iter},
        "build_phases_ms": {kk: round(v, 2) for kk, v in phases.items() if kk.endswith("_ms")},
        "build_roofline": build_roofline,
        "graph_bytes": graph.graph_bytes,
        "pops_per_query": round(cnt[0] / Q, 1), "dist_evals_per_query": round(cnt[1] / Q, 1),
        "rows_gathered_per_query": round(cnt[2] / Q, 1),
        "large_batch": large,
        "random_row_gather_ceiling_GBps": gather_ceiling,
        "curve": curve,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
