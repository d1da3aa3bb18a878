"""GPU parity of ragged_attn_padded (pack + attention + unpack of one layer in one launch) against
the fp64 oracle of the padded layout, and bit-for-bit against the three-launch path."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import binding
from paper_2604_15408_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 2e-3
_TD = {"f16": torch.float16, "bf16": torch.bfloat16}


def _padded_qkv(B, N, H, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    return tuple(torch.randn(B, N, H, 64, generator=g, dtype=torch.float32).to(_TD[dtype]) for _ in range(3))


def run_padded(q, k, v, keep, scale, fill_mode, out_dtype=None, sentinel=55.0):
    dev = "cuda:0"
    o = torch.full(q.shape, sentinel, dtype=out_dtype or q.dtype, device=dev)
    binding.ragged_attn_padded(q.to(dev), k.to(dev), v.to(dev), o, keep.to(dev), scale, fill_mode)
    torch.cuda.synchronize()
    return o.cpu()


@pytest.mark.parametrize("B,N,H,p,dtype", [
    (1, 1, 1, 1.0, "f16"), (2, 197, 3, 0.2, "f16"), (3, 197, 2, 1.0, "f16"), (4, 64, 2, 0.5, "bf16"),
    (2, 577, 2, 0.3, "f16"), (3, 300, 1, 0.02, "f16"), (2, 1100, 1, 0.1, "f16"), (5, 65, 12, 0.7, "bf16"),
])
@pytest.mark.parametrize("fill_mode", [0, 1])
def test_padded_parity(B, N, H, p, dtype, fill_mode):
    keep = wl.keep_bernoulli(B, N, p, 7 * B + N)
    if B >= 3:
        keep[1, :] = 0                                          # an image with nothing kept
    q, k, v = _padded_qkv(B, N, H, dtype, 31 * B + N)
    want = oracle.attn_padded(wl.to_words(q), wl.to_words(k), wl.to_words(v), keep.numpy(), 0.125, dtype)
    got = run_padded(q, k, v, keep, 0.125, fill_mode).to(torch.float64).numpy()
    kb = keep.numpy().astype(bool)
    err = np.abs(got[kb] - want[kb])
    bound = TOL + (np.abs(want[kb]) * 2.0 ** -8 if dtype == "bf16" else 0.0)
    assert err.size == 0 or np.all(err <= bound), f"max abs err {err.max():.3e}"
    if fill_mode == 1:
        assert not got[~kb].any()                               # dropped rows are +0
    else:
        assert np.all(got[~kb] == 55.0)                         # dropped rows untouched


def test_padded_fp32_output_and_negative_scale():
    keep = wl.keep_bernoulli(2, 150, 0.4, 3)
    q, k, v = _padded_qkv(2, 150, 2, "bf16", 4)
    want = oracle.attn_padded(wl.to_words(q), wl.to_words(k), wl.to_words(v), keep.numpy(), -0.125, "bf16")
    got = run_padded(q, k, v, keep, -0.125, 1, out_dtype=torch.float32).to(torch.float64).numpy()
    assert np.max(np.abs(got - want)) <= TOL


def test_padded_equals_pack_attend_unpack_bit_for_bit():
    """Same tiles, same order of operations: the single launch must reproduce the three-launch path
    exactly, on the headline shape."""
    w = wl.deit_b_pruned(0.2)
    dev = "cuda:0"
    B, N, H, D, C = w.B, w.N, w.H, w.D, w.C
    q, k, v = _padded_qkv(B, N, H, "f16", 99)
    keep = w.keep.to(dev)
    fused = run_padded(q, k, v, w.keep, w.scale, 1)

    cu = torch.zeros(B + 1, dtype=torch.int32, device=dev)
    gidx = torch.zeros(B * N, dtype=torch.int32, device=dev)
    packed = [torch.zeros(B * N, C, dtype=torch.float16, device=dev) for _ in range(3)]
    for src, dst in zip((q, k, v), packed):
        binding.ragged_pack(src.view(B, N, C).to(dev), keep, dst, cu, gidx)
    o = torch.zeros(B * N, H, D, dtype=torch.float16, device=dev)
    binding.ragged_attn(packed[0].view(-1, H, D), packed[1].view(-1, H, D), packed[2].view(-1, H, D),
                        o, cu, N, w.scale)
    out = torch.zeros(B, N, C, dtype=torch.float16, device=dev)
    binding.ragged_unpack(o.view(-1, C), keep, cu, gidx, out, 1)
    torch.cuda.synchronize()
    assert torch.equal(out.cpu().view(torch.int16), fused.view(B, N, C).view(torch.int16))


def test_padded_ignores_garbage_in_dropped_rows():
    keep = wl.keep_bernoulli(3, 120, 0.5, 11)
    q, k, v = _padded_qkv(3, 120, 2, "f16", 12)
    a = run_padded(q, k, v, keep, 0.125, 1)
    kb = keep.bool()
    for t in (q, k, v):
        t[~kb] = float("nan")
    b = run_padded(q, k, v, keep, 0.125, 1)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_padded_graph_replay():
    from paper_2604_15408_amd.harness import capture
    dev = "cuda:0"
    keep = wl.keep_bernoulli(4, 197, 0.3, 21)
    q, k, v = (t.to(dev) for t in _padded_qkv(4, 197, 3, "f16", 22))
    kd = keep.to(dev)
    o = torch.zeros_like(q)
    fn = lambda: binding.ragged_attn_padded(q, k, v, o, kd, 0.125, 1)
    fn()
    torch.cuda.synchronize()
    want = o.clone()
    g = capture(torch, fn)
    for _ in range(3):
        o.fill_(7.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(o.view(torch.int16), want.view(torch.int16))
