"""GPU parity of ragged_linear (bias / GELU / residual epilogues) and ragged_layernorm against the fp64
oracle.  Tolerance of the linear layer, derived from its arithmetic: products of 16-bit inputs are
exact in the fp32 accumulator; accumulating K/32 partial sums costs at most (K/32 + 1) * 2^-24 * S with
S = sum_k |x_k||w_k| (<= 2^-16 * S for K <= 8192); bias, GELU (approximation error 1.5e-7, slope <= 1.13)
and residual are applied in fp32; the single rounding to the output type is half an ulp.  Hence
|got - want| <= ulp_rel * |want| + 2^-15 * S + 1e-6, with ulp_rel = 2^-10 (fp16) or 2^-7 (bf16)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import binding
from paper_2604_15408_amd import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
_TD = {"f16": torch.float16, "bf16": torch.bfloat16}
_ULP = {"f16": 2.0 ** -10, "bf16": 2.0 ** -7}


def _rand(shape, seed, dtype, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(*shape, generator=g) * scale).to(dtype)


def check_linear(M, N, K, dtype="f16", act="none", bias=True, residual=False, rows=None, cap=None, seed=0):
    tdt = _TD[dtype]
    cap = M if cap is None else cap
    x = _rand((cap, K), 10 + seed, tdt)
    w = _rand((N, K), 20 + seed, tdt, K ** -0.5)
    b = _rand((N,), 30 + seed, tdt, 0.5) if bias else None
    r = _rand((cap, N), 40 + seed, tdt) if residual else None
    y = torch.full((cap, N), 77.0, dtype=tdt, device=DEV)
    rows_dev = None if rows is None else torch.tensor([rows], dtype=torch.int32, device=DEV)
    binding.ragged_linear(x.to(DEV), w.to(DEV), None if b is None else b.to(DEV), None if r is None else r.to(DEV),
                          y, rows_dev, act)
    torch.cuda.synchronize()
    live = cap if rows is None else min(rows, cap)
    got = y.cpu()
    assert torch.all(got[live:] == 77.0), "rows past the device row count were written"
    if live == 0:
        return 0.0
    xw, ww = wl.to_words(x[:live]), wl.to_words(w)
    want = oracle.linear(xw, ww, None if b is None else wl.to_words(b), None if r is None else wl.to_words(r[:live]),
                         act, dtype, threads=oracle.max_threads())
    absx = wl.to_words(x[:live].abs())
    absw = wl.to_words(w.abs())
    S = oracle.linear(absx, absw, dtype=dtype, threads=oracle.max_threads())
    err = np.abs(got[:live].to(torch.float64).numpy() - want)
    bound = _ULP[dtype] * np.abs(want) + 2.0 ** -15 * S + 1e-6
    assert np.all(err <= bound), (float(err.max()), float((err / bound).max()))
    return float((err / bound).max())


@pytest.mark.parametrize("M,N,K", [(1, 128, 64), (16, 128, 64), (128, 128, 128), (129, 256, 192), (300, 384, 768),
                                   (1334, 768, 768), (1000, 2304, 768), (515, 768, 3072)])
def test_linear_bias(M, N, K):
    check_linear(M, N, K)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("act,residual", [("none", False), ("gelu", False), ("none", True), ("gelu", True)])
def test_linear_epilogues(dtype, act, residual):
    check_linear(391, 384, 256, dtype, act, True, residual, seed=3)
    check_linear(70, 128, 64, dtype, act, False, residual, seed=4)


def test_linear_device_row_count():
    check_linear(640, 256, 128, rows=0)
    check_linear(640, 256, 128, rows=1)
    check_linear(640, 256, 128, rows=127)
    check_linear(640, 256, 128, rows=128)
    check_linear(640, 256, 128, rows=513)
    check_linear(640, 256, 128, rows=5000)                      # larger than the capacity: the capacity wins


def test_linear_residual_in_place_and_gelu_tails():
    tdt = torch.float16
    M, N, K = 200, 256, 128
    x, w = _rand((M, K), 1, tdt), _rand((N, K), 2, tdt, K ** -0.5)
    r = _rand((M, N), 3, tdt)
    y = r.clone().to(DEV)
    binding.ragged_linear(x.to(DEV), w.to(DEV), None, y, y)                 # y += x w^T
    torch.cuda.synchronize()
    want = oracle.linear(wl.to_words(x), wl.to_words(w), None, wl.to_words(r))
    assert np.all(np.abs(y.cpu().to(torch.float64).numpy() - want) <= 2.0 ** -10 * np.abs(want) + 1e-3)
    # GELU far into both tails: identity weights (K = N = 128), inputs spread over [-12, 12]
    t = torch.linspace(-12, 12, 128 * 64).reshape(64, 128).to(tdt)
    eye = torch.eye(128, dtype=tdt)
    out = torch.zeros(64, 128, dtype=tdt, device=DEV)
    binding.ragged_linear(t.to(DEV), eye.to(DEV), None, None, out, None, "gelu")
    torch.cuda.synchronize()
    want = oracle.linear(wl.to_words(t), wl.to_words(eye), act="gelu")
    err = np.abs(out.cpu().to(torch.float64).numpy() - want)
    assert np.all(err <= 2.0 ** -10 * np.abs(want) + 1.2e-7), float(err.max())     # fp16 subnormal spacing 6e-8


@pytest.mark.parametrize("M,C,dtype", [(1, 8, "f16"), (5, 768, "f16"), (1334, 768, "f16"), (33, 192, "bf16"),
                                       (100, 2048, "f16"), (7, 1000, "bf16")])
def test_layernorm(M, C, dtype):
    tdt = _TD[dtype]
    x = (_rand((M, C), 5, tdt, 2.0) + 0.75).to(tdt)
    g = (_rand((C,), 6, tdt, 0.3) + 1.0).to(tdt)
    b = _rand((C,), 7, tdt, 0.5)
    y = torch.zeros(M, C, dtype=tdt, device=DEV)
    binding.ragged_layernorm(x.to(DEV), g.to(DEV), b.to(DEV), y, None, 1e-6)
    torch.cuda.synchronize()
    want = oracle.layernorm(wl.to_words(x), wl.to_words(g), wl.to_words(b), 1e-6, dtype)
    err = np.abs(y.cpu().to(torch.float64).numpy() - want)
    # fp32 statistics (relative 1e-6) and one rounding to the output type
    assert np.all(err <= _ULP[dtype] * np.abs(want) + 1e-5 * (1 + np.abs(want))), float(err.max())


def test_layernorm_rows_and_in_place():
    tdt = torch.float16
    x = _rand((50, 768), 8, tdt, 3.0)
    g, b = torch.ones(768, dtype=tdt), torch.zeros(768, dtype=tdt)
    buf = x.clone().to(DEV)
    rows = torch.tensor([17], dtype=torch.int32, device=DEV)
    binding.ragged_layernorm(buf, g.to(DEV), b.to(DEV), buf, rows, 1e-6)    # in place, first 17 rows only
    torch.cuda.synchronize()
    got = buf.cpu()
    assert torch.equal(got[17:], x[17:])
    want = oracle.layernorm(wl.to_words(x[:17]), wl.to_words(g), wl.to_words(b), 1e-6)
    assert np.all(np.abs(got[:17].to(torch.float64).numpy() - want) <= 2.0 ** -10 * np.abs(want) + 2e-5)
