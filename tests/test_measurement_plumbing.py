"""The exhaustive search behind every recall figure (`exhaustive` in the package's report module, which
bench.py calls) against the oracle's plain definition, on the CPU; its two self-checks must fire when the
matrix product it relies on returns wrong rows (as a float32 product with an output beyond 2 GiB has done on
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


def test_self_checks_catch_a_wrong_product(small, monkeypatch):
    base, queries = small
    real = torch.Tensor.__matmul__

    def broken(a, b):
        out = real(a, b)
        if out.dtype == torch.float32 and out.dim() == 2 and out.shape[0] >= 8:
            out = out.clone()
            out[out.shape[0] * 3 // 4:] = 1e9  # far too large a product: distances clamp to zero
        return out

    monkeypatch.setattr(torch.Tensor, "__matmul__", broken)
    with pytest.raises(RuntimeError, match="exhaustive search"):
        report.exhaustive(torch, torch.from_numpy(base), torch.from_numpy(queries), 10, chunk=16)


def test_recall_counts_distances_within_the_kth(small):
    gt_d = torch.tensor([[1.0, 2.0, 3.0], [1.0, 1.0, 1.0]])
    found = torch.tensor([[1.0, 3.0, 9.0], [1.0, 1.0, 2.0]])
    assert abs(report.recall(found, gt_d, rel=0.0) - (2 + 2) / 6) < 1e-6
    import bench
    assert abs(bench.recall_at_k(found, gt_d) - (2 + 2) / 6) < 1e-6
