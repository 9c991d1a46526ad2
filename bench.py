#!/usr/bin/env python3
"""Benchmark of the GGNN hot path on one MI355X.

Workload of the timed region: the 1M x 128 configuration (float32 integer-valued vectors in [0,255] from a
seeded 1024-component Gaussian mixture, 10 000 queries of the same distribution, L2, K=24, k=10).  The graph
is built once on the GPU (build seconds are reported); a "step" is one search of the whole query batch at the
operating point that first reaches Recall@10 >= 0.95.  Prints one JSON line.

Beside the timed region the default run also records (each outside the timed region, each in a try block of
its own so that a failure costs that record only): the QPS-vs-recall curve of the workload, the recall of the
operating point on a fresh 100 000-query batch it was not tuned on, the for-all quality of the constructed
graph, the same workload with four levels, what each construction step buys (refinement passes, the
symmetric-linking constraint, the construction slack) with the batch-size series, and compact records (construction seconds, curve, roofline of the
search kernel) of the other workloads: 1M x 96 real-valued with k = 10 and k = 100, 1.2M x 100 cosine with
K = 40, and 10M x 128 uint8.  --quick skips them.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
import traceback

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FORMULA = ("Q*(D*e + k*8) + pops*K*4 + rows_gathered*(4 + D*e), e = bytes per element; pops and rows_gathered are "
           "counted by the kernel itself; rows actually gathered (start rows included) stand in for the method's "
           "distance evaluations: a point proposed again after it was rejected counts as an evaluation of the method "
           "but is not gathered again")


def ground_truth(torch, base, queries, k, cosine=False):
    """Exact k nearest neighbours by exhaustive search with torch (measurement plumbing, outside the timed
    region): the package's self-checking block-wise search.  On integer-valued data every float32 partial sum
    is an exact integer."""
    from paper_1912_01059_amd.report import exhaustive
    return exhaustive(torch, base, queries, k, cosine=cosine)


def recall_at_k(dists, gt_d, rel=0.0):
    """Recall@k (the paper's consensus C@k), tolerant of exact distance ties at the k-th place:
    a returned point counts if it is no farther than the k-th true neighbour (times 1 + rel for
    real-valued data, where the exhaustive search's float32 rounding differs from the library's)."""
    k = gt_d.shape[1]
    return float(((dists <= gt_d[:, k - 1:k] * (1.0 + rel)).sum(1).clamp(max=k).float().mean() / k).item())


def algorithmic_bytes(cnt_sum, Q, D, esize, K, k):
    """per launch: query vectors, one adjacency row per pop, one base row (and its id) per row gathered, results"""
    return Q * (D * esize + k * 8) + cnt_sum[0] * K * 4 + cnt_sum[2] * (4 + D * esize)


def time_point(torch, graph, queries, k, op, every, reps=3, out=None):
    """One operating point: counters from one launch, then `reps` timed launches (HIP events on the launch
    stream).  Returns (ids, dists, counter sums, ms per launch)."""
    kw = dict(pq_cap=op.get("pq_cap", 64), visited_cap=op["visited_cap"], every_layer=every)
    if out is None:
        ids, dists, cnt = graph.query(queries, k, op["beam"], op["slack"], counters=True, **kw)
    else:
        ids, dists = out
        _, _, cnt = graph.query(queries, k, op["beam"], op["slack"], counters=True, out=out, **kw)
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        graph.query(queries, k, op["beam"], op["slack"], out=(ids, dists), asynchronous=True, **kw)
    e1.record(stream)
    torch.cuda.synchronize()
    return ids, dists, cnt.double().sum(0).tolist(), e0.elapsed_time(e1) / reps


def curve_of(torch, graph, queries, k, ops, every, gt_d, rel, D, esize, K):
    """QPS-vs-recall points, each with the algorithmic rate of its launch."""
    Q = queries.shape[0]
    pts = []
    for op in ops:
        ids, dists, cs, ms = time_point(torch, graph, queries, k, op, every)
        gbps = algorithmic_bytes(cs, Q, D, esize, K, k) / (ms * 1e-3) / 1e9
        pts.append(dict(beam=op["beam"], slack=op["slack"], visited_cap=op["visited_cap"],
                        recall=round(recall_at_k(dists, gt_d, rel), 4), qps=round(Q / ms * 1e3), kernel_ms=round(ms, 3),
                        pops=round(cs[0] / Q, 1), rows_gathered=round(cs[2] / Q, 1), algorithmic_GBps=round(gbps, 1),
                        frac=round(gbps / HBM_PEAK_GBS, 4)))
    return pts


def best_point(points, bar=0.95):
    ok = [p for p in points if p["recall"] >= bar]
    return max(ok, key=lambda p: p["qps"]) if ok else None


def profile_value(key, op_tag):
    """A figure taken from a committed rocprofv3 counter summary (profiles/*_pmc.txt): only from the summary
    that names this workload, size and operating point in a line of its own (`op_tag`)."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_pmc.txt"))):
        text = open(path).read()
        if op_tag not in text.splitlines():
            continue
        for line in text.splitlines():
            if line.startswith(key + ":"):
                return float(line.split(":")[1].split()[0])
    return None


def workload_records(torch, ggnn, ggnn_inputs, name, dev, label, levels, build_iter, variants, every, n=None, gpu_gen=False,
                     large=0):
    """Compact records of another workload, one per (k, operating points) variant on one constructed graph:
    construction seconds and phases, QPS-vs-recall points with the roofline figure of each, and the fastest
    point at Recall >= 0.95 if there is one.  `large` (sets drawn on the GPU): that point again on a fresh batch
    of so many queries, with its recall measured on the first 10 000 of them."""
    cfg = dict(ggnn_inputs.CONFIGS[name])
    t0 = time.perf_counter()
    if gpu_gen:
        N = n or cfg["N"]
        base = ggnn_inputs.gmm_int_torch(N, cfg["D"], cfg["components"], cfg["sigma"], cfg["data_seed"], cfg["data_seed"] + 1,
                                         dev, cfg["dtype"])
        queries = ggnn_inputs.gmm_int_torch(cfg["Q"], cfg["D"], cfg["components"], cfg["sigma"], cfg["data_seed"],
                                            cfg["query_seed"], dev, cfg["dtype"])
    else:
        base_np, queries_np, cfg = ggnn_inputs.make(name, n=n)
        base, queries = torch.from_numpy(base_np).to(dev), torch.from_numpy(queries_np).to(dev)
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0
    N, D = base.shape
    esize, K = base.element_size(), cfg["K"]
    cosine = cfg["metric"] == "cosine"
    t0 = time.perf_counter()
    graph = ggnn.build(base, K, levels, seed=42, metric=ggnn.COSINE if cosine else ggnn.L2, visited_cap=build_iter, max_iter=build_iter)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    phases = graph.times()
    rel = 0.0 if cfg["kind"] == "gmm" else 2e-5
    e_row = 4 if cosine else esize  # a cosine graph gathers rows of its float32 unit-length copy
    recs = []
    for k, ops in variants:
        _, gt_d = ground_truth(torch, base, queries, k, cosine=cosine)
        pts = curve_of(torch, graph, queries, k, ops, every, gt_d, rel, D, e_row, K)
        recs.append({"workload": "%s: N=%d D=%d %s %s K=%d k=%d levels=%d Q=%d" % (label, N, D, cfg["dtype"], cfg["metric"], K, k,
                                                                                 levels, queries.shape[0]),
                     "data": "synthetic (%s generator, %.1f s)" % ("torch, on the GPU" if gpu_gen else "numpy", gen_s),
                     "descent": "every layer (Alg. 4)" if every else "top layer, then bottom layer (Sec. 4.4)",
                     "build_seconds": round(build_s, 3), "build_limit": build_iter,
                     "build_phases_ms": {kk: round(v, 1) for kk, v in phases.items() if kk.endswith("_ms") and kk != "total_ms"},
                     "recall_at": k, "curve": pts, "at_recall_0.95": best_point(pts)})
        if large > 0 and gpu_gen and best_point(pts):
            op = best_point(pts)
            ql = ggnn_inputs.gmm_int_torch(large, cfg["D"], cfg["components"], cfg["sigma"], cfg["data_seed"],
                                           cfg["query_seed"] + 7, dev, cfg["dtype"])
            _, ld, lcs, lms = time_point(torch, graph, ql, k, op, every)
            _, lgt = ground_truth(torch, base, ql[:10_000], k, cosine=cosine)
            lbytes = algorithmic_bytes(lcs, large, D, e_row, K, k)
            recs[-1]["large_batch"] = {"queries": large, "slack": op["slack"], "visited_cap": op["visited_cap"],
                                       "qps": round(large / lms * 1e3, 1), "kernel_ms": round(lms, 3),
                                       "algorithmic_GBps": round(lbytes / (lms * 1e-3) / 1e9, 1),
                                       "frac": round(lbytes / (lms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                       "heldout_recall": round(recall_at_k(ld[:10_000], lgt, rel), 4),
                                       "note": "fresh queries, two launches with the bottom-layer searches ordered by region; "
                                               "the algorithmic rate counts rows served by the L2 too"}
            del ql
    del graph, base, queries
    torch.cuda.empty_cache()
    return recs


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
    ap.add_argument("--quick", action="store_true", help="the timed region and its roofline only: no curve, no other workloads")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the records of the other workloads")
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
    t_start = time.perf_counter()
    cfg0 = ggnn_inputs.CONFIGS[args.workload]
    if cfg0["dtype"] == "u8" and (args.n or cfg0["N"]) >= 2_000_000:
        # too large to draw on the host in benchmark time: the same mixture drawn with torch on the GPU
        cfg = dict(cfg0, N=args.n or cfg0["N"])
        base = ggnn_inputs.gmm_int_torch(cfg["N"], cfg["D"], cfg["components"], cfg["sigma"], cfg["data_seed"],
                                         cfg["data_seed"] + 1, dev, "u8")
        queries = ggnn_inputs.gmm_int_torch(cfg["Q"], cfg["D"], cfg["components"], cfg["sigma"], cfg["data_seed"],
                                            cfg["query_seed"], dev, "u8")
        base_np = queries_np = None
    else:
        base_np, queries_np, cfg = ggnn_inputs.make(args.workload, n=args.n)
        base = torch.from_numpy(base_np).to(dev)
        queries = torch.from_numpy(queries_np).to(dev)
    N, D = base.shape
    Q, k, K = queries.shape[0], cfg["k"], cfg["K"]
    esize = base.element_size()
    metric = ggnn.COSINE if cfg["metric"] == "cosine" else ggnn.L2
    e_row = 4 if metric == ggnn.COSINE else esize
    extras = not args.quick

    # ---- construction (timed once; the graph stays resident) ----
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # a construction of minutes reports its steps on stderr (the callback waits for the stream after each step,
    # which the short constructions are spared)
    progress = None
    if N >= 20_000_000:
        def progress(step, l_top, l_m, seconds):
            print("construction: %s(%d, %d) done at %.1f s" % (step, l_top, l_m, seconds), file=sys.stderr, flush=True)
    graph = ggnn.build(base, K, args.levels, seed=42, metric=metric, visited_cap=args.build_iter, max_iter=args.build_iter,
                       progress=progress)
    torch.cuda.synchronize()
    build_s = time.perf_counter() - t0
    phases = graph.times()

    # the construction's dominant kernel (merge_kernel): adjacency rows and base rows its searches read over the
    # merge time.  This is an algorithmic rate: rows served by the L2 count too, so it is not a fraction of the
    # HBM peak; the HBM-side rate comes from hardware counters (profiles/), for the bottom-layer merge dispatch
    merge_bytes = phases["merge_pops"] * K * 4 + phases["merge_rows"] * (4 + D * e_row)
    build_tag = "build_point: %s N=%d levels=%d build_limit=%d" % (args.workload, N, args.levels, args.build_iter)
    merge_hbm = profile_value("merge_bottom_hbm_GBps", build_tag)
    build_roofline = {"kernel": "merge_kernel", "bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBS,
                      "algorithmic_GBps": round(merge_bytes / (phases["merge_ms"] * 1e-3) / 1e9, 1),
                      "hbm_GBps": merge_hbm, "frac_hbm": round(merge_hbm / HBM_PEAK_GBS, 4) if merge_hbm else None,
                      "pops": int(phases["merge_pops"]), "rows_gathered": int(phases["merge_rows"]),
                      "note": "algorithmic_GBps counts rows served by the L2 too (upper layers, rows shared by neighbouring "
                              "searches), so it may exceed the HBM peak and is not a roofline fraction; hbm_GBps / frac_hbm: "
                              "FETCH_SIZE + WRITE_SIZE of the bottom-layer merge dispatch over its duration (profiles/)"}

    errors = {}
    try:
        _, gt_d = ground_truth(torch, base, queries, k, cosine=(metric == ggnn.COSINE))
    except Exception as exc:  # no recall figure then, but the timed region and its roofline are still reported
        gt_d = None
        errors["ground_truth"] = "%s: %s" % (type(exc).__name__, exc)
        traceback.print_exc(file=sys.stderr)
    rel = 0.0 if cfg["kind"] == "gmm" else 2e-5  # integer-valued rows have exact float32 distances

    # ---- operating point (the cheapest point of the curve below that keeps Recall@10 half a point above 0.95)
    ids = torch.empty((Q, k), dtype=torch.int32, device=dev)
    dists = torch.empty((Q, k), dtype=torch.float32, device=dev)
    chosen = dict(beam=args.beam, slack=args.slack, visited_cap=args.visited_cap, pq_cap=args.pq_cap)
    every = not args.direct_drop
    kw = dict(pq_cap=chosen["pq_cap"], visited_cap=chosen["visited_cap"], every_layer=every)
    _, _, cnt = graph.query(queries, k, chosen["beam"], chosen["slack"], counters=True, out=(ids, dists), **kw)

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
    final_recall = recall_at_k(dists, gt_d, rel) if gt_d is not None else None

    # ---- roofline of the search kernel: algorithmic bytes per launch / kernel time ----
    cs = cnt.double().sum(0).tolist()
    algo_bytes = algorithmic_bytes(cs, Q, D, e_row, K, k)
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    op_tag = "operating_point: %s N=%d levels=%d beam=%d slack=%g visited_cap=%d pq_cap=%d Q=%d" % (
        args.workload, N, args.levels, chosen["beam"], chosen["slack"], chosen["visited_cap"], chosen["pq_cap"], Q)
    traffic = profile_value("traffic_bytes_per_launch", op_tag)
    traffic = int(traffic) if traffic else None
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "frac_hbm": round(traffic / (kernel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
                "kernel": "query_kernel", "kernel_ms": round(kernel_ms, 3), "algorithmic_bytes_per_launch": int(algo_bytes),
                "formula": FORMULA}

    def attempt(name, fn):
        try:
            return fn()
        except Exception as exc:  # a failed side record must not cost the benchmark line
            errors[name] = "%s: %s" % (type(exc).__name__, exc)
            traceback.print_exc(file=sys.stderr)
            return None

    # ---- QPS-vs-recall curve of the workload (10 000 queries) ----
    curve = []
    if extras:
        sweep = [dict(beam=10, slack=sl, visited_cap=v, pq_cap=64)
                 for (sl, v) in [(0.02, 40), (0.03, 40), (0.04, 48), (0.044, 48), (0.048, 48), (0.05, 56), (0.05, 64),
                                 (0.065, 96), (0.08, 128), (0.1, 192), (0.15, 384), (0.2, 512), (0.3, 1024)]]
        curve = attempt("curve", lambda: curve_of(torch, graph, queries, k, sweep, every, gt_d, rel, D, e_row, K)) or []

    # ---- steady state and held-out recall: a fresh batch large enough to keep every CU busy (the paper's own
    # batch-size study peaks near 95 000 queries); the operating point was not tuned on these queries
    large = None
    if args.large_batch > 0 and cfg["kind"] == "gmm":
        def large_batch():
            if base_np is None:
                ql = ggnn_inputs.gmm_int_torch(args.large_batch, D, cfg["components"], cfg["sigma"], cfg["data_seed"],
                                               cfg["query_seed"] + 7, dev, cfg["dtype"])
                qn = ql
            else:
                qn = ggnn_inputs.gmm_int(args.large_batch, D, cfg["components"], cfg["sigma"], cfg["data_seed"],
                                         cfg["query_seed"] + 7, cfg["dtype"])
                ql = torch.from_numpy(qn).to(dev)
            lids, ld, lcs, lms = time_point(torch, graph, ql, k, chosen, every)
            lbytes = algorithmic_bytes(lcs, len(qn), D, e_row, K, k)
            ltag = op_tag.replace("Q=%d" % Q, "Q=%d" % len(qn))
            ltraffic = profile_value("large_batch_traffic_bytes", ltag)
            rec = {"queries": len(qn), "qps": round(len(qn) / lms * 1e3, 1), "kernel_ms": round(lms, 3),
                   "algorithmic_GBps": round(lbytes / (lms * 1e-3) / 1e9, 1),
                   "traffic": int(ltraffic) if ltraffic else None,
                   "frac_hbm": round(ltraffic / (lms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if ltraffic else None,
                   "note": "two launches with the bottom-layer searches ordered by region (one part per XCD); algorithmic_GBps "
                           "counts rows served by the L2 too and is not a fraction of the HBM peak"}
            if extras:
                _, lgt = ground_truth(torch, base, ql, k)
                rec["heldout_recall_at_10"] = round(recall_at_k(ld, lgt, rel), 4)
            return rec
        large = attempt("large_batch", large_batch)

    gather_ceiling = None
    if D * esize <= 512 and metric == ggnn.L2:  # the probe reads rows of up to 512 bytes of the array as given
        def ceiling():
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
            return round(n_probe * (D * esize + 4) / (e0g.elapsed_time(e1g) / 3 * 1e-3) / 1e9, 1)
        gather_ceiling = attempt("gather_ceiling", ceiling)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- for-all quality of the constructed bottom layer (Sec. 5.2.4): C@1 / C@10 of sampled rows
    quality = None
    if extras:
        def graph_quality():
            sample = torch.arange(0, N, max(1, N // 2000), device=dev)
            gi, _ = ground_truth(torch, base, base[sample], 11, cosine=(metric == ggnn.COSINE))
            e0_, _, _ = graph.export_layer(0)
            rows = torch.from_numpy(e0_[sample.cpu().numpy()]).to(dev)
            truth = gi[:, 1:11]  # the nearest is the point itself
            c1 = (rows[:, 0:1] == truth[:, 0:1]).float().mean().item()
            c10 = (rows[:, :12, None] == truth[:, None, :]).any(1).float().sum(1).div(10).mean().item()
            return {"sample": int(sample.numel()), "c_at_1": round(c1, 4), "c_at_10": round(c10, 4),
                    "note": "first entry / first 12 entries of a row against the exact 1 / 10 nearest neighbours"}
        quality = attempt("graph_quality", graph_quality)

    # ---- the same workload with four levels (the paper's own choice) ----
    levels4 = None
    if extras and args.levels != 4 and args.workload == "sift1m":
        def four_levels():
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g4 = ggnn.build(base, K, 4, seed=42, metric=metric, visited_cap=args.build_iter, max_iter=args.build_iter)
            torch.cuda.synchronize()
            b4 = time.perf_counter() - t0
            ops = [dict(beam=b, slack=sl, visited_cap=v) for (b, sl, v) in
                   [(10, 0.03, 40), (10, 0.04, 48), (10, 0.048, 48), (10, 0.05, 64), (16, 0.04, 64), (10, 0.065, 96), (10, 0.08, 128)]]
            pts = curve_of(torch, g4, queries, k, ops, True, gt_d, rel, D, e_row, K)
            return {"build_seconds": round(b4, 3), "layers": g4.n, "curve": pts, "at_recall_0.95": best_point(pts)}
        levels4 = attempt("levels4", four_levels)

    # ---- what each construction step buys (Sec. 4.2.1, Alg. 6, Eq. 4's slack) and the batch-size series, all at
    # the timed operating point on this workload
    ablations = None
    if extras and args.workload == "sift1m":
        def ablation_records():
            def one(limit=None, **kw):
                lim = limit or args.build_iter
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ga = ggnn.build(base, K, args.levels, seed=42, metric=metric, visited_cap=lim, max_iter=lim, **kw)
                if limit:
                    kw = dict(kw, build_limit=limit)
                torch.cuda.synchronize()
                secs = time.perf_counter() - t0
                _, ad, acs, ams = time_point(torch, ga, queries, k, chosen, every)
                rec = dict(kw, build_seconds=round(secs, 3), recall_at_10=round(recall_at_k(ad, gt_d, rel), 4),
                           qps=round(Q / ams * 1e3, 1), pops_per_query=round(acs[0] / Q, 1),
                           inverse_links_per_row=round(float(ga.export_inv_count(0).mean()), 3))
                del ga
                return rec
            res = {"refinements": [one(refinements=r) for r in (0, 1, 2, 3)],
                   "sym_constraint": [one(sym_constraint=on) for on in (True, False)],
                   "tau_build": [one(tau_build=tb) for tb in (0.05, 0.1, 0.2, 0.5)],
                   "build_limit": [one(limit=v) for v in (64, 96, 128, 192, 384)]}
            reps = -(-200_000 // Q)
            big = queries.repeat(reps, 1)[torch.randperm(Q * reps, device=dev,
                                                         generator=torch.Generator(device=dev).manual_seed(5))].contiguous()
            series = []
            for nq in (100, 1000, 3000, 10_000, 30_000, 100_000, 200_000):
                _, _, _, bms = time_point(torch, graph, big[:nq].contiguous(), k, chosen, every)
                series.append({"queries": nq, "kernel_ms": round(bms, 4), "qps": round(nq / bms * 1e3, 1)})
            res["batch_size"] = series
            return res
        ablations = attempt("ablations", ablation_records)

    # ---- CPU baseline: the oracle's search of the same graph on a sample of the queries ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ggnn_ref as R
        if base_np is None:
            base_np, queries_np = base.cpu().numpy(), queries.cpu().numpy()
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
        gt_ok = bool(np.allclose(bf_d, gt_d[:16].cpu().numpy(), rtol=2e-5, atol=1e-6)) if gt_d is not None else None
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
            del sg, sb, gg
        del og

    # ---- the other workloads (compact records; their numbers are not `value`) ----
    workloads = []
    if extras and not args.no_other_workloads and args.workload == "sift1m" and args.n is None:
        graph_bytes, graph_s, graph_n = graph.graph_bytes, graph.s, graph.n
        del graph
        del base, queries
        torch.cuda.empty_cache()
        specs = [
            ("deep1m", lambda: workload_records(torch, ggnn, ggnn_inputs, "deep1m", dev, "deep1m", 4, 384,
                                                [(10, [dict(beam=10, slack=0.35, visited_cap=v) for v in (128, 256, 512, 768)]),
                                                 (100, [dict(beam=100, slack=0.35, visited_cap=v) for v in (512, 1024)])], False)),
            ("glove1m", lambda: workload_records(torch, ggnn, ggnn_inputs, "glove1m", dev, "glove1m", 4, 384,
                                                 [(10, [dict(beam=10, slack=0.35, visited_cap=v) for v in (512, 2048, 4096)])], False)),
            ("sift10m_u8", lambda: workload_records(torch, ggnn, ggnn_inputs, "sift100m_u8", dev, "10M-point subset of sift100m_u8", 4, 192,
                                                    [(10, [dict(beam=10, slack=sl, visited_cap=v) for (sl, v) in
                                                           ((0.05, 64), (0.08, 128), (0.1, 160), (0.12, 192), (0.2, 384))])], True,
                                                    n=10_000_000, gpu_gen=True, large=100_000)),
        ]
        for nm, fn in specs:
            workloads.extend(attempt(nm, fn) or [])
    else:
        graph_bytes, graph_s, graph_n = graph.graph_bytes, graph.s, graph.n

    out = {
        "metric": "queries/s at Recall@10>=0.95 (1M x 128 L2, k=10)" if args.workload == "sift1m" and args.n is None else "queries/s (workload: see config)", "value": round(qps, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if esize == 4 else "u8",
        "data": "synthetic",
        "config": {"workload": "%s: N=%d D=%d Q=%d K=%d k=%d levels=%d" % (args.workload, N, D, Q, K, k, args.levels),
                   "beam": chosen["beam"], "slack": chosen["slack"], "pq_cap": chosen["pq_cap"],
                   "visited_cap": chosen["visited_cap"], "descent": "every layer (Alg. 4)" if every else "top layer, then bottom layer (Sec. 4.4)"},
        "recall_at_10": round(final_recall, 4) if final_recall is not None else None,
        "heldout_recall_at_10": (large or {}).get("heldout_recall_at_10"),
        "build_seconds": round(build_s, 3),
        "build_config": {"levels": args.levels, "K": K, "segment_size": graph_s, "tau_build": 0.5, "refinements": 2,
                         "pq_cap": 64, "visited_cap": args.build_iter, "max_iter": args.build_iter},
        "build_phases_ms": {kk: round(v, 2) for kk, v in phases.items() if kk.endswith("_ms")},
        "build_roofline": build_roofline,
        "graph_bytes": graph_bytes, "layers": graph_n,
        "graph_quality": quality,
        "pops_per_query": round(cs[0] / Q, 1), "dist_evals_per_query": round(cs[1] / Q, 1),
        "rows_gathered_per_query": round(cs[2] / Q, 1),
        "large_batch": large,
        "random_row_gather_ceiling_GBps": gather_ceiling,
        "curve": curve,
        "levels4": levels4,
        "ablations": ablations,
        "workloads": workloads,
        "errors": errors or None,
        "bench_seconds": round(time.perf_counter() - t_start, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
