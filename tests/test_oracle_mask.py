"""Pins of the oracle's keep-mask producer (squared l2 token scores, per-image top-k with the class
token always kept): NumPy norms / stable sort, closed forms, invariants, planted mistakes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import workloads as wl


def _x(B, N, C, seed, dtype=torch.float16):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(B, N, C, generator=g).to(dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_scores_equal_numpy_sum_of_squares(dtype):
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    x = _x(3, 17, 40, 1, tdt)
    got = oracle.scores_l2(wl.to_words(x), dtype)
    xd = x.to(torch.float64).numpy()
    assert np.allclose(got, (xd * xd).sum(-1), rtol=1e-15, atol=0)
    assert np.allclose(np.sqrt(got), np.linalg.norm(xd, axis=-1), rtol=1e-15)
    # small integers: every square and every partial sum is exact
    xi = torch.randint(-8, 9, (2, 5, 12), generator=torch.Generator().manual_seed(2)).to(tdt)
    assert np.array_equal(oracle.scores_l2(wl.to_words(xi), dtype), (xi.to(torch.int64) ** 2).sum(-1).numpy())


def _numpy_topk(scores, k):
    B, N = scores.shape
    keep = np.zeros((B, N), dtype=np.uint8)
    keep[:, 0] = 1
    for i in range(B):
        order = 1 + np.argsort(-scores[i, 1:], kind="stable")          # ties keep position order
        keep[i, order[: max(0, min(k - 1, N - 1))]] = 1
    return keep


@pytest.mark.parametrize("B,N,k", [(1, 1, 1), (2, 9, 1), (3, 9, 4), (4, 197, 40), (2, 197, 197), (2, 50, 500), (3, 64, 2)])
def test_topk_equals_stable_argsort(B, N, k):
    rng = np.random.default_rng(B * 100 + N + k)
    scores = rng.random((B, N))
    got = oracle.keep_topk(scores, k)
    assert np.array_equal(got, _numpy_topk(scores, k))
    assert np.all(got[:, 0] == 1) and np.all(got.sum(1) == min(k, N))


def test_topk_ties_and_closed_forms():
    # all scores equal: CLS plus the first k-1 other positions
    same = np.ones((2, 10))
    assert oracle.keep_topk(same, 4).tolist() == [[1, 1, 1, 1, 0, 0, 0, 0, 0, 0]] * 2
    # increasing scores: CLS plus the last k-1
    inc = np.arange(10, dtype=np.float64)[None, :]
    assert oracle.keep_topk(inc, 4).tolist() == [[1, 0, 0, 0, 0, 0, 0, 1, 1, 1]]
    # a huge CLS score does not take a slot away from the others, a tiny one is kept anyway
    s = np.array([[100.0, 1, 5, 3, 4], [-1.0, 1, 5, 3, 4]])
    assert oracle.keep_topk(s, 3).tolist() == [[1, 0, 1, 0, 1]] * 2
    # groups of ties across the cut: positions decide
    t = np.array([[0.0, 2, 2, 2, 1, 2]])
    assert oracle.keep_topk(t, 3).tolist() == [[1, 1, 1, 0, 0, 0]]
    # images are independent
    rng = np.random.default_rng(5)
    a, b = rng.random((1, 30)), rng.random((1, 30))
    both = oracle.keep_topk(np.concatenate([a, b]), 7)
    assert np.array_equal(both[0:1], oracle.keep_topk(a, 7)) and np.array_equal(both[1:2], oracle.keep_topk(b, 7))


def test_scores_then_topk_on_feature_rows_and_planted_mistakes():
    x = _x(4, 60, 32, 7)
    scores = oracle.scores_l2(wl.to_words(x))
    keep = oracle.keep_topk(scores, 15)
    xd = x.to(torch.float64).numpy()
    norms = np.linalg.norm(xd, axis=-1)
    for i in range(4):
        kept, dropped = norms[i, 1:][keep[i, 1:] == 1], norms[i, 1:][keep[i, 1:] == 0]
        assert kept.size == 14 and kept.min() >= dropped.max()
    wrong = {
        "smallest norms kept": _numpy_topk(-scores, 15),
        "l1 norm": _numpy_topk(np.abs(xd).sum(-1), 15),
        "class token competes": np.stack([(np.argsort(np.argsort(-s, kind="stable"), kind="stable") < 15) for s in scores]).astype(np.uint8),
        "k instead of k-1 others": _numpy_topk(scores, 16),
    }
    for name, bad in wrong.items():
        assert not np.array_equal(keep, bad), name
