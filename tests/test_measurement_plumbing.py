"""The exhaustive search behind every recall figure (`exhaustive` in the package's report module, which
bench.py calls) against the oracle's plain definition, on the CPU; its two self-checks must act when the
matrix product it relies on returns wrong values (as a float32 product with an output beyond 2 GiB has done on
the GPU), and the recall measure must count what it says."""
import numpy as np
import pytest
import torch

import ggnn_inputs
from oracle import ggnn_ref as R
from paper_1912_01059_amd import report


@pytest.fixture(scope="module")
def small():
    base, queries, _ = ggnn_inputs.make("sift10k", n=3000, q=40)
    return base, queries


@pytest.mark.parametrize("cosine", [False, True])
def test_exhaustive_search_equals_the_oracles(small, cosine):
    base, queries = small
    ids, d = report.exhaustive(torch, torch.from_numpy(base), torch.from_numpy(queries), 10, cosine=cosine, chunk=16)
    gt, gt_d = R.bruteforce(base, queries, 10, metric=R.COSINE if cosine else R.L2)
    assert np.allclose(d.numpy(), gt_d, rtol=2e-5, atol=2e-6)
    # ids agree wherever the distances of the row are distinct (equal distances may swap)
    distinct = np.all(np.diff(gt_d, axis=1) > (5e-6 if cosine else 1e-3), axis=1)
    assert distinct.sum() >= 20
    assert np.array_equal(ids.numpy()[distinct], gt[distinct])


def test_blocks_stay_under_the_limit(small, monkeypatch):
    base, queries = small
    seen = []
    real = torch.topk

    def spy(x, *a, **kw):
        seen.append(x.numel())
        return real(x, *a, **kw)

    monkeypatch.setattr(report, "MAX_BLOCK_ELEMS", 16 * 500)
    monkeypatch.setattr(torch, "topk", spy)
    ids, d = report.exhaustive(torch, torch.from_numpy(base), torch.from_numpy(queries), 10, chunk=16)
    monkeypatch.undo()
    assert max(seen) == 16 * 500  # distance blocks of 16 x 500 (the plain scans and the merges of partial results are smaller)
    _, gt_d = R.bruteforce(base, queries, 10)
    assert np.allclose(d.numpy(), gt_d, rtol=2e-5, atol=2e-6)


def test_wrong_rows_of_the_product_are_searched_again_without_it(small, monkeypatch, capfd):
    """Rows of the product that are far too large (their distances clamp to zero, as seen on the GPU): the
    recomputation of the reported distances notices, the block is searched again without a product, and the
    result is still the oracle's."""
    base, queries = small
    real = torch.Tensor.__matmul__

    def broken(a, b):
        out = real(a, b)
        if out.dtype == torch.float32 and out.dim() == 2 and out.shape[0] >= 8:
            out = out.clone()
            out[out.shape[0] * 3 // 4:] = 1e9
        return out

    monkeypatch.setattr(torch.Tensor, "__matmul__", broken)
    ids, d = report.exhaustive(torch, torch.from_numpy(base), torch.from_numpy(queries), 10, chunk=16)
    monkeypatch.undo()
    assert "searching them again without it" in capfd.readouterr().err
    _, gt_d = R.bruteforce(base, queries, 10)
    assert np.allclose(d.numpy(), gt_d, rtol=2e-5, atol=2e-6)


def test_neighbours_hidden_by_the_product_are_caught_by_the_plain_scan(small, monkeypatch):
    """Columns of the product that are far too small make half of the base points look far away: every reported
    distance is right, but true neighbours are missing.  The scan without a product over a few queries raises."""
    base, queries = small
    real = torch.Tensor.__matmul__

    def broken(a, b):
        out = real(a, b)
        if out.dtype == torch.float32 and out.dim() == 2 and out.shape[1] >= 64:
            out = out.clone()
            out[:, ::2] = -1e9
        return out

    monkeypatch.setattr(torch.Tensor, "__matmul__", broken)
    with pytest.raises(RuntimeError, match="plain scan"):
        report.exhaustive(torch, torch.from_numpy(base), torch.from_numpy(queries), 10, chunk=16)


def test_recall_counts_distances_within_the_kth(small):
    gt_d = torch.tensor([[1.0, 2.0, 3.0], [1.0, 1.0, 1.0]])
    found = torch.tensor([[1.0, 3.0, 9.0], [1.0, 1.0, 2.0]])
    assert abs(report.recall(found, gt_d, rel=0.0) - (2 + 2) / 6) < 1e-6
    import bench
    assert abs(bench.recall_at_k(found, gt_d) - (2 + 2) / 6) < 1e-6


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_follow_the_stated_formula():
    import bench
    # 3 queries of 128 float32 elements, k = 10, K = 24: 7 pops and 50 rows gathered in all
    want = 3 * (128 * 4 + 10 * 8) + 7 * 24 * 4 + 50 * (4 + 128 * 4)
    assert bench.algorithmic_bytes([7, 60, 50, 0], 3, 128, 4, 24, 10) == want
    assert "rows_gathered*(4 + D*e)" in bench.FORMULA and "pops*K*4" in bench.FORMULA


def test_best_point_is_the_fastest_at_the_recall_bar():
    import bench
    pts = [dict(recall=0.94, qps=30), dict(recall=0.951, qps=20), dict(recall=0.97, qps=10)]
    assert bench.best_point(pts)["qps"] == 20
    assert bench.best_point(pts[:1]) is None


def test_profile_figures_are_only_taken_for_the_operating_point_they_name(tmp_path, monkeypatch):
    import bench
    (tmp_path / "profiles").mkdir()
    (tmp_path / "profiles" / "a_pmc.txt").write_text("operating_point: w N=10 Q=10000 slack=0.048\ntraffic_bytes_per_launch: 3520000000 bytes\n")
    (tmp_path / "profiles" / "b_pmc.txt").write_text("operating_point: w N=20 Q=10000 slack=0.048\ntraffic_bytes_per_launch: 99 bytes\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.profile_value("traffic_bytes_per_launch", "operating_point: w N=10 Q=10000 slack=0.048") == 3.52e9
    assert bench.profile_value("traffic_bytes_per_launch", "operating_point: w N=20 Q=10000 slack=0.048") == 99.0
    assert bench.profile_value("traffic_bytes_per_launch", "operating_point: w N=10 Q=10000 slack=0.05") is None
    assert bench.profile_value("traffic_bytes_per_launch", "operating_point: w N=1") is None  # whole lines only
    assert bench.profile_value("no_such_key", "operating_point: w N=10 Q=10000 slack=0.048") is None


def test_committed_counter_summaries_name_their_operating_points():
    """The benchmark's own workload finds its HBM traffic figures in profiles/ (the tags are whole lines)."""
    import bench
    tag = "operating_point: sift1m N=1000000 levels=3 beam=10 slack=0.048 visited_cap=48 pq_cap=64 Q=10000"
    assert bench.profile_value("traffic_bytes_per_launch", tag) > 1e9
    assert bench.profile_value("large_batch_traffic_bytes", tag.replace("Q=10000", "Q=100000")) > 1e9
    assert bench.profile_value("merge_bottom_hbm_GBps", "build_point: sift1m N=1000000 levels=3 build_limit=192") > 1000
