"""GPU parity of ragged_pack / ragged_unpack against the CPU oracle: bit-exact, every byte."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _features(B, N, C, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(B, N, C, generator=g, dtype=torch.float32)
    return x.to(torch.float16 if dtype == "f16" else torch.bfloat16)


def check_pack(x_cpu, keep_cpu, cap=None):
    B, N, C = x_cpu.shape
    xw = wl.to_words(x_cpu)
    want_packed, want_cu, want_gidx = oracle.pack(xw, keep_cpu.numpy())
    T = int(want_cu[-1])
    packed, cu, gidx = hp.gpu_pack(x_cpu, keep_cpu, cap)
    cap = B * N if cap is None else cap
    kept = min(T, cap)
    assert np.array_equal(cu, want_cu)
    assert np.array_equal(gidx[:kept], want_gidx[:kept])
    assert np.array_equal(packed[:kept], want_packed[:kept])
    assert np.all(gidx[kept:] == -7), "gather_idx written past T"
    assert np.all(packed[kept:] == hp.SENTINEL), "packed rows written past T"
    return want_packed, want_cu, want_gidx


@pytest.mark.parametrize("B,N,C,p,dtype", [
    (1, 1, 8, 1.0, "f16"), (1, 7, 64, 0.5, "f16"), (2, 64, 64, 0.5, "bf16"), (3, 65, 192, 0.3, "f16"),
    (5, 197, 192, 0.2, "f16"), (4, 577, 768, 0.3, "f16"), (7, 130, 24, 1.0, "bf16"), (6, 33, 768, 0.0, "f16"),
    (32, 197, 768, 0.2, "f16"), (64, 197, 768, 0.7, "f16"), (3, 1000, 64, 0.05, "f16"),
    # masks beyond 16 KB (the prefix count runs its remainder passes) and chunks of 16, 32 and 64 tokens
    (100, 197, 64, 0.3, "f16"), (400, 197, 8, 0.5, "bf16"), (700, 197, 8, 0.2, "f16"),
])
def test_pack_bit_exact(B, N, C, p, dtype):
    keep = wl.keep_bernoulli(B, N, p, 11 * B + N)
    if p == 0.0:
        keep[:, 0] = 0                                   # an all-dropped batch
        keep[B // 2, N // 2] = 1                         # ... but for one token
    check_pack(_features(B, N, C, dtype, 5), keep)


def test_pack_tiny_workload_closed_form():
    w = wl.tiny()
    _, cu, gidx = check_pack(w.features(), w.keep)
    assert cu.tolist() == [0, 197, 237] and gidx[197] == 197


def test_pack_all_dropped_and_empty_images():
    x = _features(4, 50, 64, "f16", 1)
    keep = torch.zeros(4, 50, dtype=torch.uint8)
    check_pack(x, keep)                                   # T = 0
    keep[1, [0, 49]] = 1
    keep[3, 17] = 1
    check_pack(x, keep)                                   # images 0 and 2 empty


def test_pack_nonzero_bytes_and_bool_masks():
    x = _features(3, 40, 64, "f16", 2)
    keep = wl.keep_bernoulli(3, 40, 0.5, 3)
    loud = keep * torch.randint(1, 256, keep.shape, dtype=torch.int64,
                                generator=torch.Generator().manual_seed(1)).to(torch.uint8)
    a = check_pack(x, loud)
    b = check_pack(x, keep.bool().to(torch.uint8))
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
    packed, cu, gidx = hp.gpu_pack(x, keep.bool())        # torch.bool goes through the binding too
    assert np.array_equal(cu, a[1])


def test_pack_unaligned_mask_pointer():
    """The mask may start at any byte address (a slice of a larger mask)."""
    B, N, C = 5, 197, 64
    x = _features(B, N, C, "f16", 3)
    big = wl.keep_bernoulli(1, B * N + 3, 0.4, 9).reshape(-1)
    keep_cpu = big[3:].reshape(B, N).clone()
    dev = "cuda:0"
    keep_dev = big.to(dev)[3:].view(B, N)                 # data_ptr offset by 3 bytes
    assert keep_dev.data_ptr() % 16 == 3 and keep_dev.is_contiguous()
    from paper_2604_15408_amd import binding
    packed = torch.zeros(B * N, C, dtype=torch.float16, device=dev)
    cu = torch.zeros(B + 1, dtype=torch.int32, device=dev)
    gidx = torch.zeros(B * N, dtype=torch.int32, device=dev)
    binding.ragged_pack(x.to(dev), keep_dev, packed, cu, gidx)
    torch.cuda.synchronize()
    want_packed, want_cu, want_gidx = oracle.pack(wl.to_words(x), keep_cpu.numpy())
    T = int(want_cu[-1])
    assert np.array_equal(cu.cpu().numpy(), want_cu)
    assert np.array_equal(gidx.cpu().numpy()[:T], want_gidx)
    assert np.array_equal(hp.words(packed)[:T], want_packed)


def test_pack_capacity_clamps_writes():
    x = _features(4, 60, 64, "f16", 4)
    keep = wl.keep_bernoulli(4, 60, 0.8, 5)
    check_pack(x, keep, cap=37)


@pytest.mark.parametrize("fill_mode", [0, 1])
@pytest.mark.parametrize("B,N,C,p,dtype", [
    (1, 1, 8, 1.0, "f16"), (2, 64, 64, 0.5, "bf16"), (3, 65, 192, 0.3, "f16"), (4, 577, 768, 0.3, "f16"),
    (32, 197, 768, 0.2, "f16"), (64, 197, 768, 0.7, "f16"), (5, 100, 64, 0.0, "f16"), (7, 130, 24, 1.0, "bf16"),
    (200, 197, 64, 0.3, "f16"), (700, 197, 8, 0.2, "f16"),      # chunks of 16 and 64 tokens in the zero-filling form
])
def test_unpack_bit_exact(B, N, C, p, dtype, fill_mode):
    keep = wl.keep_bernoulli(B, N, p, 13 * B + N)
    if p == 0.0:
        keep[:, 0] = 0
    _, cu, gidx = oracle.pack(np.zeros((B, N, 8), dtype=np.uint16), keep.numpy())
    T = int(cu[-1])
    src = _features(1, max(T, 1), C, dtype, 6)[0][:T]
    if T == 0:
        src = torch.zeros(1, C, dtype=src.dtype)          # a valid pointer; no row is read
    init = np.full((B, N, C), hp.SENTINEL, dtype=np.uint16)
    want = oracle.unpack(wl.to_words(src)[:T], keep.numpy(), cu, C, fill_mode, out_init=init)
    got = hp.gpu_unpack(src, keep, cu, gidx if T else np.zeros(1, np.int32), B, N, fill_mode)
    assert np.array_equal(got, want)
    got = hp.gpu_unpack(src, keep, cu, gidx if T else np.zeros(1, np.int32), B, N, fill_mode,
                        pass_unused=False)                # the unused argument may be NULL
    assert np.array_equal(got, want)


def test_pack_then_unpack_is_identity_on_kept_tokens():
    w = wl.deit_b_pruned(0.2)
    x = w.features()
    packed, cu, gidx = hp.gpu_pack(x, w.keep)
    T = int(cu[-1])
    src = torch.from_numpy(packed[:T].view(np.int16)).view(torch.float16)
    out = hp.gpu_unpack(src, w.keep, cu, gidx[:T].copy(), w.B, w.N, 1)
    kb = w.keep.numpy().astype(bool)
    xw = wl.to_words(x)
    assert np.array_equal(out[kb], xw[kb]) and not out[~kb].any()
