"""GPU parity of ragged_pack_attn_unpack (pack + attention + unpack of one layer in ONE launch): every
output equals what the three separate entry points produce (bit for bit), and matches the CPU
oracle's three stages (pack / unpack bit-exact, attention within the attention tolerance)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import binding
from paper_2604_15408_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 2e-3


def run_step(w, fill_mode, dtype=torch.float16, seed=0):
    """Returns the GPU buffers after one fused launch and after the three-launch path on the same inputs."""
    B, N, C, H, D = w.B, w.N, w.C, w.H, w.D
    cap = B * N
    tdt = dtype
    x = w.features().to(tdt).to(DEV)
    keep = w.keep.to(DEV)
    g = torch.Generator().manual_seed(1234 + seed)
    q, k, v = (torch.randn(cap, H, D, generator=g).to(tdt).to(DEV) for _ in range(3))

    def fresh():
        return dict(packed=torch.full((cap, C), hp.SENTINEL, dtype=torch.int16, device=DEV).view(tdt),
                    cu=torch.full((B + 1,), -7, dtype=torch.int32, device=DEV),
                    gidx=torch.full((cap,), -7, dtype=torch.int32, device=DEV),
                    o=torch.full((cap, H, D), hp.SENTINEL, dtype=torch.int16, device=DEV).view(tdt),
                    out=torch.full((B, N, C), hp.SENTINEL, dtype=torch.int16, device=DEV).view(tdt))

    one = fresh()
    binding.ragged_pack_attn_unpack(x, keep, q, k, v, one["packed"], one["cu"], one["gidx"], one["o"], one["out"],
                                    w.scale, fill_mode)
    three = fresh()
    binding.ragged_pack(x, keep, three["packed"], three["cu"], three["gidx"])
    binding.ragged_attn(q, k, v, three["o"], three["cu"], N, w.scale)
    binding.ragged_unpack(three["o"].view(cap, C), keep, three["cu"], three["gidx"], three["out"], fill_mode)
    torch.cuda.synchronize()
    return x, (q, k, v), one, three


def check(w, fill_mode, dtype=torch.float16, oracle_attn=True):
    x, (q, k, v), one, three = run_step(w, fill_mode, dtype)
    for name in ("packed", "cu", "gidx", "o", "out"):
        a, b = one[name], three[name]
        if a.dtype in (torch.float16, torch.bfloat16):
            a, b = a.view(torch.int16), b.view(torch.int16)
        assert torch.equal(a, b), f"{name} differs from the three-launch path"
    # oracle: the three stages on the same inputs
    T = w.T
    xw = wl.to_words(x.cpu())
    want_packed, want_cu, want_gidx = oracle.pack(xw, w.keep.numpy())
    assert np.array_equal(one["cu"].cpu().numpy(), want_cu)
    assert np.array_equal(one["gidx"][:T].cpu().numpy(), want_gidx)
    assert np.array_equal(hp.words(one["packed"][:T]), want_packed)
    assert torch.all(one["gidx"][T:] == -7) and np.all(hp.words(one["packed"][T:]) == hp.SENTINEL)
    assert np.all(hp.words(one["o"][T:]) == hp.SENTINEL), "o rows past T were written"
    o_words = hp.words(one["o"][:T]).reshape(T, w.C)
    init = np.full((w.B, w.N, w.C), hp.SENTINEL, dtype=np.uint16)
    want_out = oracle.unpack(o_words, w.keep.numpy(), want_cu, w.C, fill_mode, out_init=init)
    assert np.array_equal(hp.words(one["out"]), want_out)
    if oracle_attn and T > 0:
        name = "f16" if dtype == torch.float16 else "bf16"
        want_o = oracle.attn(wl.to_words(q[:T].cpu()), wl.to_words(k[:T].cpu()), wl.to_words(v[:T].cpu()), want_cu,
                             w.scale, name, threads=oracle.max_threads())
        got = one["o"][:T].cpu().to(torch.float64).numpy()
        bound = TOL + (np.abs(want_o) * 2.0 ** -8 if dtype == torch.bfloat16 else 0.0)
        assert np.all(np.abs(got - want_o) <= bound), np.max(np.abs(got - want_o))


@pytest.mark.parametrize("fill_mode", [0, 1])
def test_tiny_and_headline(fill_mode):
    check(wl.tiny(), fill_mode)
    check(wl.deit_b_pruned(0.2, 32, "f16", 1001), fill_mode)


@pytest.mark.parametrize("p,B,dtype", [(1.0, 8, torch.float16), (0.6, 16, torch.bfloat16), (0.1, 32, torch.float16),
                                       (0.4, 5, torch.bfloat16)])
def test_pruning_ratios(p, B, dtype):
    check(wl.deit_b_pruned(p, B, "f16", 77), 1, dtype)


def test_serving_384_and_empty_images():
    check(wl.serving_384(4), 1)
    B, N = 6, 197
    keep = wl.keep_bernoulli(B, N, 0.3, 5)
    keep[0] = 0
    keep[3] = 0
    keep[5] = 0
    keep[5, 196] = 1
    check(wl.Workload("holes", B, N, 12, 64, "f16", 31, keep), 1)
    check(wl.Workload("holes", B, N, 12, 64, "f16", 31, keep), 0)
    check(wl.Workload("nothing", 3, 50, 2, 64, "f16", 32, torch.zeros(3, 50, dtype=torch.uint8)), 1)


def test_masks_beyond_16_kb():
    """From B*N > 16384 mask bytes on, the count of the kept tokens in front of an image runs its remainder
    passes (q-tile 0 under the first barrier, the other q-tiles after it): 100 images of 197 tokens, lengths
    around 59 (one q-tile) and around 118 (two)."""
    check(wl.Workload("b100", 100, 197, 2, 64, "f16", 35, wl.keep_bernoulli(100, 197, 0.3, 12)), 1)
    check(wl.Workload("b100w", 100, 197, 1, 64, "f16", 36, wl.keep_bernoulli(100, 197, 0.6, 13)), 0)


def test_small_heads_and_odd_sizes():
    keep = wl.keep_bernoulli(7, 65, 0.5, 9)
    check(wl.Workload("odd", 7, 65, 1, 64, "f16", 33, keep), 0)
    keep = wl.keep_bernoulli(3, 1000, 0.2, 10)
    check(wl.Workload("long", 3, 1000, 3, 64, "f16", 34, keep), 1)


@pytest.mark.parametrize("seed", range(12))
def test_random_batches(seed):
    """Seeded random geometry, keep probability, dtype and fill mode, with images that keep nothing and
    batches whose class tokens are not forced."""
    g = torch.Generator().manual_seed(7000 + seed)
    ri = lambda lo, hi: int(torch.randint(lo, hi + 1, (1,), generator=g))
    B, N, H = ri(1, 12), ri(1, 400), ri(1, 6)
    p = [0.0, 0.05, 0.2, 0.5, 0.9, 1.0][ri(0, 5)]
    keep = (torch.rand(B, N, generator=g) < p).to(torch.uint8)
    if ri(0, 1):
        keep[:, 0] = 1
    if ri(0, 3) == 0:
        keep[ri(0, B - 1)] = 0
    check(wl.Workload(f"random{seed}", B, N, H, 64, "f16", 500 + seed, keep), ri(0, 1),
          [torch.float16, torch.bfloat16][ri(0, 1)])


def test_graph_replays_match_eager():
    from paper_2604_15408_amd.harness import capture
    w = wl.deit_b_pruned(0.3, 8)
    B, N, C, H, D = w.B, w.N, w.C, w.H, w.D
    cap = B * N
    x = w.features().to(DEV)
    keep = w.keep.to(DEV)
    g = torch.Generator().manual_seed(5)
    q, k, v = (torch.randn(cap, H, D, generator=g).to(torch.float16).to(DEV) for _ in range(3))
    bufs = dict(packed=torch.zeros(cap, C, dtype=torch.float16, device=DEV),
                cu=torch.zeros(B + 1, dtype=torch.int32, device=DEV),
                gidx=torch.zeros(cap, dtype=torch.int32, device=DEV),
                o=torch.zeros(cap, H, D, dtype=torch.float16, device=DEV),
                out=torch.zeros(B, N, C, dtype=torch.float16, device=DEV))

    def step():
        binding.ragged_pack_attn_unpack(x, keep, q, k, v, bufs["packed"], bufs["cu"], bufs["gidx"], bufs["o"],
                                        bufs["out"], w.scale, 1)
    step()
    torch.cuda.synchronize()
    want = {n: t.clone() for n, t in bufs.items()}
    graph = capture(torch, step)
    for rep in range(3):
        for t in bufs.values():
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, t in bufs.items():
            a, b = (t.view(torch.int16), want[n].view(torch.int16)) if t.dtype == torch.float16 else (t, want[n])
            assert torch.equal(a, b), n


def test_prepared_calls_reproduce_checked_calls():
    """Every pre-marshalled call (what the benchmark's fastest modes issue) gives the checked call's result."""
    from paper_2604_15408_amd.harness import PaddedPath, Path
    w = wl.deit_b_pruned(0.3, B=6)
    p = Path(w, fill_mode=1)
    p.step()
    torch.cuda.synchronize()
    want = {n: getattr(p, n).clone() for n in ("packed", "cu", "gidx", "o", "out")}

    def same():
        T = w.T
        assert torch.equal(p.cu, want["cu"]) and torch.equal(p.gidx[:T], want["gidx"][:T])
        for n in ("packed", "o"):
            assert torch.equal(getattr(p, n)[:T].view(torch.int16), want[n][:T].view(torch.int16)), n
        assert torch.equal(p.out.view(torch.int16), want["out"].view(torch.int16))

    for make in (p.prepared_step, p.prepared_one_launch):
        for n in ("packed", "o", "out"):
            getattr(p, n).zero_()
        p.cu.zero_()
        call = make()
        call()
        torch.cuda.synchronize()
        same()
    pad = PaddedPath(w, 1)
    pad.run()
    torch.cuda.synchronize()
    ref = pad.o.clone()
    pad.o.zero_()
    pad.prepared()()
    torch.cuda.synchronize()
    assert torch.equal(pad.o.view(torch.int16), ref.view(torch.int16))
    # the remaining prepare_* helpers
    x = torch.randn(40, 128, device=DEV).half()
    wgt = torch.randn(128, 128, device=DEV).half()
    y1, y2 = torch.zeros(40, 128, device=DEV).half(), torch.zeros(40, 128, device=DEV).half()
    binding.ragged_linear(x, wgt, None, None, y1)
    binding.prepare_linear(x, wgt, None, None, y2)()
    g, bta = torch.ones(128, device=DEV).half(), torch.zeros(128, device=DEV).half()
    n1, n2 = torch.zeros_like(x), torch.zeros_like(x)
    binding.ragged_layernorm(x, g, bta, n1)
    binding.prepare_layernorm(x, g, bta, n2)()
    cu = torch.tensor([0, 10, 40], dtype=torch.int32, device=DEV)
    c1, c2 = torch.zeros(2, 128, device=DEV).half(), torch.zeros(2, 128, device=DEV).half()
    binding.ragged_cls_extract(x, cu, c1)
    binding.prepare_cls_extract(x, cu, c2)()
    keep_rows = (torch.arange(40, device=DEV) % 3 != 0).to(torch.uint8)
    outs = []
    for fn in (binding.ragged_repack, lambda *a: binding.prepare_repack(*a)()):
        po, co, go = torch.zeros_like(x), torch.zeros_like(cu), torch.zeros(40, dtype=torch.int32, device=DEV)
        fn(x, keep_rows, cu, po, co, go)
        outs.append((po, co, go))
    qkv = torch.randn(40, 3, 2, 64, device=DEV).half()
    o1, o2 = torch.zeros(40, 2, 64, device=DEV).half(), torch.zeros(40, 2, 64, device=DEV).half()
    binding.ragged_attn_strided(qkv[:, 0], qkv[:, 1], qkv[:, 2], o1, cu, 30, 0.125)
    binding.prepare_attn_strided(qkv[:, 0], qkv[:, 1], qkv[:, 2], o2, cu, 30, 0.125)()
    torch.cuda.synchronize()
    assert torch.equal(y1, y2) and torch.equal(n1, n2) and torch.equal(c1, c2) and torch.equal(o1, o2)
    assert all(torch.equal(a, b) for a, b in zip(*outs))


def test_steps_on_three_streams_fill_every_buffer_set():
    """The benchmark's multi-stream mode: steps issued round-robin on three streams, each with its own
    buffers, leave in every buffer set exactly what a single step leaves."""
    from paper_2604_15408_amd.harness import Path, StreamedSteps
    w = wl.deit_b_pruned(0.25, B=9, seed=4)
    ref = Path(w, fill_mode=1)
    ref.one_launch()
    torch.cuda.synchronize()
    ms = StreamedSteps(w, fill_mode=1, streams=3)
    for p in ms.paths:
        for n in ("packed", "o", "out"):
            getattr(p, n).fill_(float("nan"))
        p.cu.fill_(-1)
    torch.cuda.synchronize()
    for _ in range(7):                                  # 7 steps: sets 0, 1, 2, 0, 1, 2, 0
        ms.step()
    torch.cuda.synchronize()
    T = w.T
    for p in ms.paths:
        assert torch.equal(p.cu, ref.cu) and torch.equal(p.gidx[:T], ref.gidx[:T])
        for n in ("packed", "o"):
            assert torch.equal(getattr(p, n)[:T].view(torch.int16), getattr(ref, n)[:T].view(torch.int16)), n
        assert torch.equal(p.out.view(torch.int16), ref.out.view(torch.int16))
