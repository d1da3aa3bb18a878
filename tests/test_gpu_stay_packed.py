"""GPU parity of the stay-packed pieces against the CPU oracle: packed-to-packed re-pack and CLS
extraction are bit-exact; attention on strided token rows matches the oracle within the attention
tolerance and is bit-identical to the contiguous entry point."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import binding
from paper_2604_15408_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ATTN_TOL = 2e-3            # max |GPU - fp64 oracle| for unit-variance inputs, as for ragged_attn


def _rows(T, C, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(T, C, generator=g).to(torch.float16 if dtype == "f16" else torch.bfloat16)


def _lengths(B, n_max, seed, empties=()):
    g = torch.Generator().manual_seed(seed)
    n = torch.randint(1, n_max + 1, (B,), generator=g).tolist()
    for i in empties:
        n[i] = 0
    return n


def gpu_repack(rows_cpu, keep_rows_cpu, cu_np, cap_in=None, cap_out=None):
    T, C = rows_cpu.shape
    B = cu_np.size - 1
    cap_in = max(T, 1) if cap_in is None else cap_in
    cap_out = cap_in if cap_out is None else cap_out
    src = torch.full((cap_in, C), float("nan"), dtype=rows_cpu.dtype)
    src[:T] = rows_cpu
    kr = torch.ones(cap_in, dtype=torch.uint8)            # bytes past T are set: they must be ignored
    kr[:T] = keep_rows_cpu
    dst = torch.full((cap_out, C), hp.SENTINEL, dtype=torch.int16, device=DEV).view(rows_cpu.dtype)
    cu_out = torch.full((B + 1,), -7, dtype=torch.int32, device=DEV)
    gi = torch.full((cap_out,), -7, dtype=torch.int32, device=DEV)
    binding.ragged_repack(src.to(DEV), kr.to(DEV), torch.from_numpy(cu_np).to(DEV), dst, cu_out, gi)
    torch.cuda.synchronize()
    return hp.words(dst), cu_out.cpu().numpy(), gi.cpu().numpy()


def check_repack(rows_cpu, keep_rows_cpu, cu_np, cap_in=None, cap_out=None):
    want_rows, want_cu, want_gi = oracle.repack(wl.to_words(rows_cpu), keep_rows_cpu.numpy(), cu_np)
    got_rows, got_cu, got_gi = gpu_repack(rows_cpu, keep_rows_cpu, cu_np, cap_in, cap_out)
    kept = min(int(want_cu[-1]), got_rows.shape[0])
    assert np.array_equal(got_cu, want_cu)
    assert np.array_equal(got_gi[:kept], want_gi[:kept])
    assert np.array_equal(got_rows[:kept], want_rows[:kept])
    assert np.all(got_gi[kept:] == -7) and np.all(got_rows[kept:] == hp.SENTINEL)
    return want_rows, want_cu, want_gi


@pytest.mark.parametrize("B,n_max,C,p,dtype,empties", [
    (1, 1, 8, 1.0, "f16", ()), (3, 9, 64, 0.5, "f16", ()), (5, 70, 192, 0.5, "bf16", (0, 3)),
    (32, 60, 768, 0.6, "f16", (7,)), (64, 197, 768, 0.7, "f16", (0, 1, 63)), (64, 197, 768, 0.0, "f16", ()),
    (6, 577, 768, 0.3, "f16", (5,)), (300, 197, 64, 0.5, "f16", (10, 11, 12)), (2, 1000, 24, 1.0, "bf16", ()),
])
def test_repack_bit_exact(B, n_max, C, p, dtype, empties):
    n = _lengths(B, n_max, 3 * B + n_max, empties)
    cu = hp.cu_from_lengths(n)
    T = int(cu[-1])
    keep_rows = wl.keep_bernoulli(1, T, p, B + 1).reshape(-1)
    check_repack(_rows(T, C, dtype, 9), keep_rows, cu)


def test_repack_spare_capacity_and_small_output():
    n = _lengths(9, 40, 2, (4,))
    cu = hp.cu_from_lengths(n)
    T = int(cu[-1])
    rows = _rows(T, 64, "f16", 4)
    keep_rows = wl.keep_bernoulli(1, T, 0.5, 5).reshape(-1)
    check_repack(rows, keep_rows, cu, cap_in=T + 129)          # chunk starts beyond T exist and exit
    check_repack(rows, keep_rows, cu, cap_in=T + 3, cap_out=7)  # overflow rows dropped, counts still true
    check_repack(rows, keep_rows, cu, cap_in=2 * T + 64)


def test_repack_no_rows_at_all():
    cu = np.zeros(5, dtype=np.int32)
    rows = _rows(0, 64, "f16", 1)
    got_rows, got_cu, got_gi = gpu_repack(rows, torch.zeros(0, dtype=torch.uint8), cu, cap_in=20)
    assert got_cu.tolist() == [0] * 5 and np.all(got_gi == -7) and np.all(got_rows == hp.SENTINEL)


def test_repack_of_pack_is_pack_of_both_masks():
    """Two-stage pruning kept packed == one pack with the AND of the masks (the same identity pins the oracle)."""
    w = wl.deit_b_pruned(keep_prob=0.7, B=16, dtype="f16", seed=3)
    x = w.features()
    B, N, C = x.shape
    packed1, cu1, gi1 = hp.gpu_pack(x, w.keep)
    T1 = int(cu1[-1])
    second = wl.keep_bernoulli(B, N, 0.5, 77)
    keep_rows = second.reshape(-1)[torch.from_numpy(gi1[:T1]).long()]
    rows1 = torch.from_numpy(packed1[:T1].copy()).view(torch.float16)
    got_rows, got_cu, got_gi = gpu_repack(rows1, keep_rows, cu1)
    want_rows, want_cu, want_gi = oracle.pack(wl.to_words(x), (w.keep & second).numpy())
    T2 = int(want_cu[-1])
    assert np.array_equal(got_cu, want_cu)
    assert np.array_equal(got_rows[:T2], want_rows)
    assert np.array_equal(gi1[got_gi[:T2]], want_gi)            # composed gather index reaches the padded tensor


@pytest.mark.parametrize("B,n_max,C,dtype,empties", [
    (1, 1, 8, "f16", ()), (7, 50, 64, "bf16", (0, 6)), (64, 197, 768, "f16", (5,)), (257, 30, 192, "f16", (100,)),
])
def test_cls_extract_bit_exact(B, n_max, C, dtype, empties):
    n = _lengths(B, n_max, B, empties)
    cu = hp.cu_from_lengths(n)
    rows = _rows(int(cu[-1]), C, dtype, 8)
    want = oracle.cls_extract(wl.to_words(rows), cu)
    out = torch.full((B, C), hp.SENTINEL, dtype=torch.int16, device=DEV).view(rows.dtype)
    src = rows.to(DEV) if rows.shape[0] else torch.zeros(1, C, dtype=rows.dtype, device=DEV)
    binding.ragged_cls_extract(src, torch.from_numpy(cu).to(DEV), out)
    torch.cuda.synchronize()
    assert np.array_equal(hp.words(out), want)


@pytest.mark.parametrize("B,n_max,H,dtype,out_dtype,slots,o_pad", [
    (3, 40, 2, "f16", torch.float16, 3, 0), (8, 197, 12, "f16", torch.float16, 3, 0),
    (5, 130, 3, "bf16", torch.bfloat16, 3, 64), (4, 70, 6, "f16", torch.float32, 4, 4),
    (2, 300, 1, "bf16", torch.float32, 3, 0),
])
def test_attn_on_fused_qkv_buffer(B, n_max, H, dtype, out_dtype, slots, o_pad):
    """q, k, v are slices of one [T, slots, H, D] buffer (the layout a QKV projection writes)."""
    D = 64
    n = _lengths(B, n_max, 5 * B + H, (1,) if B > 2 else ())
    cu = hp.cu_from_lengths(n)
    T = int(cu[-1])
    tdt = torch.float16 if dtype == "f16" else torch.bfloat16
    g = torch.Generator().manual_seed(17)
    qkv_cpu = torch.randn(T, slots, H, D, generator=g).to(tdt)
    qkv = qkv_cpu.to(DEV)
    q, k, v = qkv[:, 0], qkv[:, 1], qkv[:, 2]
    o_buf = torch.full((T, H * D + o_pad), 77.0, dtype=out_dtype, device=DEV)
    o = o_buf[:, :H * D].view(T, H, D) if o_pad == 0 else o_buf.as_strided((T, H, D), (H * D + o_pad, D, 1))
    scale = D ** -0.5
    cu_dev = torch.from_numpy(cu).to(DEV)
    binding.ragged_attn_strided(q, k, v, o, cu_dev, max(n), scale)
    # contiguous entry point on de-interleaved copies: must agree bit for bit
    o2 = torch.empty(T, H, D, dtype=out_dtype, device=DEV)
    binding.ragged_attn(q.contiguous(), k.contiguous(), v.contiguous(), o2, cu_dev, max(n), scale)
    torch.cuda.synchronize()
    assert torch.equal(o.contiguous().cpu(), o2.cpu())
    if o_pad:
        assert torch.all(o_buf[:, H * D:] == 77.0), "padding between output tokens was written"
    want = oracle.attn(wl.to_words(qkv_cpu[:, 0].contiguous()), wl.to_words(qkv_cpu[:, 1].contiguous()),
                       wl.to_words(qkv_cpu[:, 2].contiguous()), cu, scale, dtype, threads=oracle.max_threads())
    err = np.abs(o.cpu().to(torch.float64).numpy() - want)
    # a bf16 output adds its own final rounding: half an ulp <= 2^-8 |o|
    bound = ATTN_TOL + (np.abs(want) * 2.0 ** -8 if out_dtype == torch.bfloat16 else 0.0)
    assert np.all(err <= bound), err.max()


def test_binding_rejects_scattered_head_block():
    qkv = torch.zeros(10, 2, 3, 64, dtype=torch.float16, device=DEV)          # [T, H, 3, D]: heads not adjacent
    bad = qkv[:, :, 0]
    o = torch.zeros(10, 2, 64, dtype=torch.float16, device=DEV)
    cu = torch.tensor([0, 10], dtype=torch.int32, device=DEV)
    with pytest.raises(ValueError):
        binding.ragged_attn_strided(bad, bad, bad, o, cu, 10, 0.125)
