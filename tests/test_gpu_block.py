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


def check_linear(M, N, K, dtype="f16", act="none", bias=True, residual=False, rows=None, cap=None, seed=0, hint=0):
    tdt = _TD[dtype]
    cap = M if cap is None else cap
    x = _rand((cap, K), 10 + seed, tdt)
    w = _rand((N, K), 20 + seed, tdt, K ** -0.5)
    b = _rand((N,), 30 + seed, tdt, 0.5) if bias else None
    r = _rand((cap, N), 40 + seed, tdt) if residual else None
    y = torch.full((cap, N), 77.0, dtype=tdt, device=DEV)
    rows_dev = None if rows is None else torch.tensor([rows], dtype=torch.int32, device=DEV)
    binding.ragged_linear(x.to(DEV), w.to(DEV), None if b is None else b.to(DEV), None if r is None else r.to(DEV),
                          y, rows_dev, act, rows_hint=hint)
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


@pytest.mark.parametrize("dtype,act,residual", [("f16", "none", False), ("bf16", "gelu", True)])
def test_linear_every_launch_shape(dtype, act, residual):
    """The launch shape follows the expected row count (the capacity, or the caller's hint): 256 x 256
    tiles for many rows or a long k-loop, 64 x 64 tiles with the k-loop split in two for few rows, 128 x 128
    tiles between.  Large capacities with a small device row count keep the oracle's work small."""
    kw = dict(dtype=dtype, act=act, residual=residual)
    check_linear(700, 1024, 256, rows=700, cap=26000, seed=5, **kw)               # 408 tiles of 256 x 256
    check_linear(300, 1024, 2048, rows=300, cap=8200, seed=6, **kw)               # long k-loop, 132 such tiles
    check_linear(700, 1024, 256, rows=700, cap=26000, seed=5, hint=3000, **kw)    # 192 tiles of 128 x 128
    check_linear(700, 1024, 256, rows=700, cap=26000, seed=5, hint=700, **kw)     # 64 x 64 tiles, k split
    check_linear(130, 128, 3072, seed=7, **kw)                                    # 64 x 64 tiles, 24 k-steps per half
    check_linear(700, 1024, 192, rows=650, cap=800, seed=8, hint=650, **kw)       # odd number of k-steps: no split


@pytest.mark.parametrize("M", [12608, 6304])
@pytest.mark.parametrize("N,K,act,residual", [(2304, 768, "none", False), (768, 768, "none", True),
                                               (3072, 768, "gelu", False), (768, 3072, "none", True)])
def test_linear_layer_shapes_at_full_size_on_sampled_rows(M, N, K, act, residual):
    """The four linear layers of a DeiT-B block at the row counts the benchmarks run (B*N for B = 64 and 32):
    the whole launch runs on the GPU, the oracle checks a sample of rows -- the first and last row of the
    buffer, rows around tile boundaries of every launch shape, and seeded random ones."""
    tdt = torch.float16
    x = _rand((M, K), 50, tdt)
    w = _rand((N, K), 51, tdt, K ** -0.5)
    b = _rand((N,), 52, tdt, 0.5)
    r = _rand((M, N), 53, tdt) if residual else None
    y = torch.full((M, N), 77.0, dtype=tdt, device=DEV)
    binding.ragged_linear(x.to(DEV), w.to(DEV), b.to(DEV), None if r is None else r.to(DEV), y, None, act)
    torch.cuda.synchronize()
    g = torch.Generator().manual_seed(M + N)
    rows = {0, 1, 63, 64, 127, 128, 255, 256, 257, M // 2, M - 257, M - 256, M - 129, M - 128, M - 65, M - 64, M - 2, M - 1}
    rows |= {int(v) for v in torch.randint(0, M, (78,), generator=g)}
    rows = sorted(rows)
    xs = x[rows]
    want = oracle.linear(wl.to_words(xs), wl.to_words(w), wl.to_words(b), None if r is None else wl.to_words(r[rows]),
                         act, "f16", threads=oracle.max_threads())
    S = oracle.linear(wl.to_words(xs.abs()), wl.to_words(w.abs()), dtype="f16", threads=oracle.max_threads())
    got = y[rows].cpu().to(torch.float64).numpy()
    bound = _ULP["f16"] * np.abs(want) + 2.0 ** -15 * S + 1e-6
    assert np.all(np.abs(got - want) <= bound), float((np.abs(got - want) / bound).max())
    assert not torch.any(y == 77.0), "some output element was never written"


@pytest.mark.parametrize("seed", range(10))
def test_linear_random_shapes(seed):
    """Seeded random problems: rows, capacity, device row count, hint, N, K, epilogue and dtype all vary."""
    g = torch.Generator().manual_seed(9000 + seed)
    ri = lambda lo, hi: int(torch.randint(lo, hi + 1, (1,), generator=g))
    cap = ri(1, 900)
    rows = [None, ri(0, cap), cap + 5][ri(0, 2)]
    live = cap if rows is None else min(rows, cap)
    hint = [0, max(1, live), cap][ri(0, 2)]
    N, K = 128 * ri(1, 6), 64 * ri(1, 14)
    check_linear(cap, N, K, dtype=["f16", "bf16"][ri(0, 1)], act=["none", "gelu"][ri(0, 1)], bias=bool(ri(0, 1)),
                 residual=bool(ri(0, 1)), rows=rows, cap=cap, seed=seed, hint=hint)


@pytest.mark.parametrize("M,N,K,act", [(500, 192, 192, "none"), (237, 576, 192, "none"), (1000, 768, 192, "gelu"),
                                        (300, 192, 768, "none"), (65, 64, 64, "none"), (130, 320, 128, "gelu")])
def test_linear_feature_counts_that_are_odd_multiples_of_64(M, N, K, act):
    """Widths of the DeiT-Tiny blocks (C = 192: 192, 576, 768) and other odd multiples of 64."""
    check_linear(M, N, K, act=act, residual=True, seed=11)
    check_linear(M, N, K, dtype="bf16", act=act, bias=False, seed=12)


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


def test_packed_block_stage_by_stage_against_the_oracle():
    """One encoder block on packed rows: every launch is checked against the oracle applied to the GPU's
    own input of that launch (so rounding of intermediate activations is not compared twice)."""
    from paper_2604_15408_amd.harness import LN_EPS, PackedBlocks
    from tests import helpers as hp
    w = wl.deit_b_pruned(0.35, B=3, dtype="f16", seed=91)
    pb = PackedBlocks(w, depth=1)
    T, C, H, D = w.T, w.C, w.H, w.D
    p = {k: wl.to_words(v.cpu()) for k, v in pb.params[0].items()}
    words = lambda t: wl.to_words(t[:T].reshape(T, -1).cpu())
    f64 = lambda t: t[:T].reshape(T, -1).cpu().to(torch.float64).numpy()
    threads = oracle.max_threads()

    def close(got, want, S=None, rel=2.0 ** -10):
        bound = rel * np.abs(want) + 1e-5 * (1 + np.abs(want)) + (0 if S is None else 2.0 ** -15 * S)
        assert np.all(np.abs(got - want) <= bound), float(np.max(np.abs(got - want) / bound))

    def lin(xin, wk, bk, res=None, act="none"):
        want = oracle.linear(xin, p[wk], p[bk], res, act, "f16", threads=threads)
        S = oracle.linear(wl.to_words(torch.from_numpy(xin.view(np.float16)).abs()),
                          wl.to_words(torch.from_numpy(p[wk].view(np.float16)).abs()), dtype="f16", threads=threads)
        return want, S

    b = pb.b
    b.ragged_pack(pb.x_in, pb.keep, pb.x, pb.cu, pb.gidx)
    torch.cuda.synchronize()
    assert int(pb.cu[-1]) == T
    x0 = words(pb.x)
    b.ragged_layernorm(pb.x, pb.params[0]["ln1_g"], pb.params[0]["ln1_b"], pb.h, pb.rows, LN_EPS)
    torch.cuda.synchronize()
    close(f64(pb.h), oracle.layernorm(x0, p["ln1_g"], p["ln1_b"], LN_EPS))
    h1 = words(pb.h)
    b.ragged_linear(pb.h, pb.params[0]["w_qkv"], pb.params[0]["b_qkv"], None, pb.qkv.view(pb.cap, 3 * C), pb.rows)
    torch.cuda.synchronize()
    close(f64(pb.qkv), *lin(h1, "w_qkv", "b_qkv"))
    qkv = pb.qkv[:T].cpu()
    b.ragged_attn_strided(pb.qkv[:, 0], pb.qkv[:, 1], pb.qkv[:, 2], pb.a, pb.cu, w.N, w.scale)
    torch.cuda.synchronize()
    want_a = oracle.attn(wl.to_words(qkv[:, 0].contiguous()), wl.to_words(qkv[:, 1].contiguous()),
                         wl.to_words(qkv[:, 2].contiguous()), hp.cu_from_lengths(w.lengths), w.scale, "f16", threads=threads)
    got_a = pb.a[:T].cpu().to(torch.float64).numpy()
    vmax = float(qkv[:, 2].abs().max())
    assert np.max(np.abs(got_a - want_a)) <= 2e-3 * max(1.0, vmax)      # the attention bar, scaled by |v|
    a_w = words(pb.a)
    b.ragged_linear(pb.a.view(pb.cap, C), pb.params[0]["w_o"], pb.params[0]["b_o"], pb.x, pb.x, pb.rows)
    torch.cuda.synchronize()
    want, S = lin(a_w, "w_o", "b_o", x0)
    close(f64(pb.x), want, S)
    x1 = words(pb.x)
    b.ragged_layernorm(pb.x, pb.params[0]["ln2_g"], pb.params[0]["ln2_b"], pb.h, pb.rows, LN_EPS)
    torch.cuda.synchronize()
    close(f64(pb.h), oracle.layernorm(x1, p["ln2_g"], p["ln2_b"], LN_EPS))
    h2 = words(pb.h)
    b.ragged_linear(pb.h, pb.params[0]["w_fc1"], pb.params[0]["b_fc1"], None, pb.mid, pb.rows, "gelu")
    torch.cuda.synchronize()
    want, S = lin(h2, "w_fc1", "b_fc1", None, "gelu")
    close(f64(pb.mid), want, S)
    mid = words(pb.mid)
    b.ragged_linear(pb.mid, pb.params[0]["w_fc2"], pb.params[0]["b_fc2"], pb.x, pb.x, pb.rows)
    torch.cuda.synchronize()
    want, S = lin(mid, "w_fc2", "b_fc2", x1)
    close(f64(pb.x), want, S)
    # rows past T of every buffer were never written
    assert not pb.x[T:].any() and not pb.mid[T:].any() and not pb.qkv[T:].any()
    # the whole loop (pack + block + CLS) in a graph reproduces the eager result
    from paper_2604_15408_amd.harness import capture
    pb.run()
    torch.cuda.synchronize()
    want_x, want_cls = pb.x.clone(), pb.cls.clone()
    g = capture(torch, pb.run)
    for _ in range(2):
        pb.x.zero_(); pb.cls.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(pb.x.view(torch.int16), want_x.view(torch.int16))
        assert torch.equal(pb.cls.view(torch.int16), want_cls.view(torch.int16))
    assert np.array_equal(wl.to_words(pb.cls.cpu()), oracle.cls_extract(words(pb.x), hp.cu_from_lengths(w.lengths)))
