"""GPU parity of the keep-mask producer: fp64 scores agree with the oracle to rounding-order level,
the top-k mask is bit-exact, and the mask feeds ragged_pack to uniform lengths."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import binding
from paper_2604_15408_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _x(B, N, C, seed, dtype=torch.float16):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(B, N, C, generator=g).to(dtype)


def gpu_mask(x, k):
    B, N, C = x.shape
    scores = torch.full((B, N), -1.0, dtype=torch.float64, device=DEV)
    keep = torch.full((B, N), 9, dtype=torch.uint8, device=DEV)
    binding.ragged_token_scores_l2(x.to(DEV), scores)
    binding.ragged_keep_topk(scores, k, keep)
    torch.cuda.synchronize()
    return scores.cpu().numpy(), keep.cpu().numpy()


@pytest.mark.parametrize("B,N,C,k,dtype", [(1, 1, 8, 1, "f16"), (3, 9, 64, 4, "f16"), (32, 197, 768, 40, "f16"),
                                           (8, 577, 768, 150, "f16"), (5, 197, 192, 197, "bf16"), (2, 1536, 64, 300, "bf16"),
                                           (4, 65, 24, 1, "f16"), (3, 50, 768, 999, "f16")])
def test_scores_and_topk(B, N, C, k, dtype):
    x = _x(B, N, C, 3 * B + N, torch.float16 if dtype == "f16" else torch.bfloat16)
    scores, keep = gpu_mask(x, k)
    want_scores = oracle.scores_l2(wl.to_words(x), dtype)
    assert np.allclose(scores, want_scores, rtol=1e-14, atol=0)
    assert np.array_equal(keep, oracle.keep_topk(scores, k))            # the decision, given the scores
    assert np.array_equal(keep, oracle.keep_topk(want_scores, k))       # and end to end
    assert np.all(keep.sum(1) == min(k, N)) and np.all(keep[:, 0] == 1)


def test_exact_scores_and_ties():
    """Small-integer features: every score is an exact integer on both sides, ties are frequent."""
    g = torch.Generator().manual_seed(4)
    x = torch.randint(-3, 4, (6, 130, 16), generator=g).to(torch.float16)
    scores, keep = gpu_mask(x, 33)
    want = oracle.scores_l2(wl.to_words(x))
    assert np.array_equal(scores, want)
    assert np.array_equal(keep, oracle.keep_topk(want, 33))
    dup = torch.ones(2, 40, 8, dtype=torch.float16)                     # all tokens identical
    _, keep = gpu_mask(dup, 5)
    assert keep.tolist() == [[1] * 5 + [0] * 35] * 2


def test_topk_on_arbitrary_scores():
    rng = np.random.default_rng(8)
    s = rng.standard_normal((7, 300))
    s[3, 10:20] = s[3, 5]                                               # a block of ties
    keep = torch.zeros(7, 300, dtype=torch.uint8, device=DEV)
    binding.ragged_keep_topk(torch.from_numpy(s).to(DEV), 60, keep)
    torch.cuda.synchronize()
    assert np.array_equal(keep.cpu().numpy(), oracle.keep_topk(s, 60))


def test_mask_feeds_pack_to_uniform_lengths():
    B, N, C, k = 32, 197, 768, 40
    x = _x(B, N, C, 11)
    xd = x.to(DEV)
    scores = torch.zeros(B, N, dtype=torch.float64, device=DEV)
    keep = torch.zeros(B, N, dtype=torch.uint8, device=DEV)
    packed = torch.zeros(B * N, C, dtype=torch.float16, device=DEV)
    cu = torch.zeros(B + 1, dtype=torch.int32, device=DEV)
    gidx = torch.zeros(B * N, dtype=torch.int32, device=DEV)
    binding.ragged_token_scores_l2(xd, scores)
    binding.ragged_keep_topk(scores, k, keep)
    binding.ragged_pack(xd, keep, packed, cu, gidx)
    torch.cuda.synchronize()
    assert cu.cpu().tolist() == [k * i for i in range(B + 1)]
    want_packed, want_cu, want_gidx = oracle.pack(wl.to_words(x), oracle.keep_topk(oracle.scores_l2(wl.to_words(x)), k))
    assert np.array_equal(wl.to_words(packed[: B * k].cpu()), want_packed)
    assert np.array_equal(gidx[: B * k].cpu().numpy(), want_gidx)
