"""Pins of the oracle's linear layer (with GELU / residual epilogues) and LayerNorm: independent
NumPy / torch float64 evaluations, closed forms, invariants, and planted mistakes that must fail."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import workloads as wl


def _rand(shape, seed, dtype=torch.float16, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(*shape, generator=g) * scale).to(dtype)


def _f64(t):
    return t.to(torch.float64).numpy()


@pytest.mark.parametrize("M,N,K,dtype", [(5, 7, 8, "f16"), (33, 48, 64, "bf16"), (17, 130, 96, "f16")])
def test_linear_matches_numpy_matmul(M, N, K, dtype):
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    x, w, b, r = _rand((M, K), 1, tdt), _rand((N, K), 2, tdt, 0.2), _rand((N,), 3, tdt), _rand((M, N), 4, tdt)
    xw, ww, bw, rw = (wl.to_words(t) for t in (x, w, b, r))
    z = _f64(x) @ _f64(w).T
    assert np.allclose(oracle.linear(xw, ww, dtype=dtype), z, rtol=1e-13, atol=1e-13)
    assert np.allclose(oracle.linear(xw, ww, bw, dtype=dtype), z + _f64(b), rtol=1e-13, atol=1e-13)
    assert np.allclose(oracle.linear(xw, ww, bw, rw, dtype=dtype), z + _f64(b) + _f64(r), rtol=1e-13, atol=1e-13)
    # GELU applies to the biased pre-activation, the residual is added after it
    t = torch.from_numpy(z + _f64(b))
    want = torch.nn.functional.gelu(t).numpy() + _f64(r)
    assert np.allclose(oracle.linear(xw, ww, bw, rw, act="gelu", dtype=dtype), want, rtol=1e-12, atol=1e-12)
    assert np.allclose(oracle.linear(xw, ww, bw, rw, act="gelu", dtype=dtype, threads=4), want, rtol=1e-12, atol=1e-12)


def test_linear_closed_forms():
    K = 16
    x = _rand((6, K), 5)
    eye = torch.eye(K, dtype=torch.float16)
    assert np.array_equal(oracle.linear(wl.to_words(x), wl.to_words(eye)), _f64(x))          # identity weights
    perm = torch.randperm(K, generator=torch.Generator().manual_seed(1))
    assert np.array_equal(oracle.linear(wl.to_words(x), wl.to_words(eye[perm])), _f64(x)[:, perm.numpy()])
    w = torch.zeros(3, K, dtype=torch.float16)
    w[0, 2], w[1, 5], w[2, 5] = 2.0, -1.0, 0.5                                                   # row n picks column k
    want = np.stack([2 * _f64(x)[:, 2], -_f64(x)[:, 5], 0.5 * _f64(x)[:, 5]], axis=1)
    assert np.array_equal(oracle.linear(wl.to_words(x), wl.to_words(w)), want)


def test_gelu_known_values():
    """GELU(t) = t * Phi(t): checked against math.erf and the textbook values at 0, +-1, +-3."""
    ts = torch.tensor([[0.0, 1.0, -1.0, 3.0, -3.0, 0.5, -0.25, 8.0, -8.0]], dtype=torch.float16)
    one = torch.ones(1, 1, dtype=torch.float16)
    got = oracle.linear(wl.to_words(ts.T.contiguous()), wl.to_words(one), act="gelu")[:, 0]
    want = [t * 0.5 * (1 + math.erf(t / math.sqrt(2))) for t in ts[0].tolist()]
    assert np.allclose(got, want, rtol=1e-14, atol=1e-300)
    assert got[0] == 0.0 and abs(got[1] - 0.8413447460685429) < 1e-15 and abs(got[2] + 0.15865525393145707) < 1e-15
    assert abs(got[7] - 8.0) < 1e-14 and abs(got[8]) < 1e-14
    assert np.allclose(got[1] - got[2], 1.0)                    # GELU(t) - GELU(-t) = t


def test_linear_planted_mistakes_are_caught():
    M, N, K = 8, 8, 8
    x, w, b, r = _rand((M, K), 7), _rand((N, K), 8), _rand((N,), 9), _rand((M, N), 10)
    good = oracle.linear(*(wl.to_words(t) for t in (x, w, b, r)), act="gelu")
    z = _f64(x) @ _f64(w).T + _f64(b)
    gelu = lambda t: torch.nn.functional.gelu(torch.from_numpy(t)).numpy()
    wrong = {
        "transposed weights": gelu(_f64(x) @ _f64(w) + _f64(b)) + _f64(r),
        "bias dropped": gelu(_f64(x) @ _f64(w).T) + _f64(r),
        "residual inside the activation": gelu(z + _f64(r)),
        "tanh form of GELU": torch.nn.functional.gelu(torch.from_numpy(z), approximate="tanh").numpy() + _f64(r),
        "bias indexed by row": gelu(_f64(x) @ _f64(w).T + _f64(b)[:, None]) + _f64(r),
    }
    for name, bad in wrong.items():
        assert np.max(np.abs(good - bad)) > 1e-4, name


@pytest.mark.parametrize("M,C,dtype", [(4, 8, "f16"), (19, 768, "f16"), (7, 192, "bf16")])
def test_layernorm_matches_torch_float64(M, C, dtype):
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    x, g, b = _rand((M, C), 11, tdt, 3.0) + 1.5, _rand((C,), 12, tdt) + 1.0, _rand((C,), 13, tdt)
    x = x.to(tdt)
    g = g.to(tdt)
    want = torch.nn.functional.layer_norm(x.to(torch.float64), (C,), g.to(torch.float64), b.to(torch.float64), 1e-6)
    got = oracle.layernorm(wl.to_words(x), wl.to_words(g), wl.to_words(b), 1e-6, dtype)
    assert np.allclose(got, want.numpy(), rtol=1e-12, atol=1e-12)


def test_layernorm_invariants_and_special_cases():
    C = 64
    x = _rand((5, C), 14, scale=2.0)
    ones, zeros = torch.ones(C, dtype=torch.float16), torch.zeros(C, dtype=torch.float16)
    y = oracle.layernorm(wl.to_words(x), wl.to_words(ones), wl.to_words(zeros), 0.0)
    assert np.allclose(y.mean(axis=1), 0.0, atol=1e-14) and np.allclose((y * y).mean(axis=1), 1.0, rtol=1e-13)
    # shift and positive scale of a row leave the normalised row unchanged (eps = 0; powers of two keep fp16 exact)
    y2 = oracle.layernorm(wl.to_words((x * 4).to(torch.float16)), wl.to_words(ones), wl.to_words(zeros), 0.0)
    assert np.allclose(y, y2, rtol=1e-13, atol=1e-13)
    # a two-element row: (a, b) -> (-1, +1) * sign(b - a)
    two = torch.tensor([[1.0, 3.0], [5.0, -2.0]], dtype=torch.float16)
    y3 = oracle.layernorm(wl.to_words(two), wl.to_words(ones[:2]), wl.to_words(zeros[:2]), 0.0)
    assert np.allclose(y3, [[-1.0, 1.0], [1.0, -1.0]], rtol=1e-15)
    # eps enters under the square root: a constant row gives beta exactly, and eps = 3 with var = 1 halves the scale
    const = torch.full((1, C), 2.5, dtype=torch.float16)
    beta = _rand((C,), 15)
    assert np.array_equal(oracle.layernorm(wl.to_words(const), wl.to_words(ones), wl.to_words(beta), 1e-6),
                          _f64(beta)[None, :])
    y4 = oracle.layernorm(wl.to_words(two), wl.to_words(ones[:2]), wl.to_words(zeros[:2]), 3.0)
    assert np.allclose(y4, [[-0.5, 0.5], [7 / math.sqrt(12.25 + 3) / 2, -7 / math.sqrt(12.25 + 3) / 2]], rtol=1e-14)


def test_layernorm_planted_mistakes_are_caught():
    M, C = 6, 32
    x, g, b = _rand((M, C), 16, scale=2.0), _rand((C,), 17) + 1.0, _rand((C,), 18)
    g = g.to(torch.float16)
    good = oracle.layernorm(wl.to_words(x), wl.to_words(g), wl.to_words(b), 1e-6)
    xd, gd, bd = _f64(x), _f64(g), _f64(b)
    mu, var = xd.mean(1, keepdims=True), xd.var(1, keepdims=True)
    wrong = {
        "unbiased variance": (xd - mu) / np.sqrt(xd.var(1, ddof=1, keepdims=True) + 1e-6) * gd + bd,
        "mean not removed": xd / np.sqrt(var + 1e-6) * gd + bd,
        "gamma and beta swapped": (xd - mu) / np.sqrt(var + 1e-6) * bd + gd,
        "normalised over rows": (xd - xd.mean(0)) / np.sqrt(xd.var(0) + 1e-6) * gd + bd,
        "eps outside the root": (xd - mu) / (np.sqrt(var) + 1e-1) * gd + bd,
    }
    for name, bad in wrong.items():
        assert np.max(np.abs(good - bad)) > 1e-3, name
