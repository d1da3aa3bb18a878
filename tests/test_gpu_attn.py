"""GPU parity of ragged_attn against the fp64 CPU oracle.

Bar: max-abs-error <= 2e-3 on N(0,1) inputs (fp16 in/out, fp16->fp32, bf16->fp32).  With bf16
OUTPUT the final rounding alone is up to half a bf16 ulp = 2^-9 * 2^floor(log2|o|) <= 2^-8 * |o|,
so that case is held to 2e-3 + 2^-8 * |oracle|.  Several outputs are correct (the reduction order
is free), so the comparison is a tolerance, never bit equality -- except where the mathematics
fixes the bits (n = 1, ragged isolation, run-to-run determinism, untouched rows).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import workloads as wl
from tests import helpers as hp

pytestmark = pytest.mark.gpu

TOL = 2e-3
_TD = {"f16": torch.float16, "bf16": torch.bfloat16}


def _qkv(T, H, dtype, seed, D=64):
    g = torch.Generator().manual_seed(seed)
    return tuple(torch.randn(T, H, D, generator=g, dtype=torch.float32).to(_TD[dtype]) for _ in range(3))


def check(lengths, H, dtype, seed, scale=0.125, out_dtype=None, max_seqlen=None, tol=TOL):
    cu = hp.cu_from_lengths(lengths)
    T = int(cu[-1])
    q, k, v = _qkv(T, H, dtype, seed)
    want = oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), cu, scale, dtype, threads=8)
    ms = max(max(lengths), 1) if max_seqlen is None else max_seqlen
    got, raw = hp.gpu_attn(q, k, v, cu, ms, scale, out_dtype, extra_rows=3)
    assert np.all(raw[T:].to(torch.float64).numpy() == 77.0), "rows past T were written"
    assert np.all(np.isfinite(got[:T]))
    err = np.abs(got[:T] - want)
    bound = tol + (np.abs(want) * 2.0 ** -8 if raw.dtype == torch.bfloat16 else 0.0)
    assert np.all(err <= bound), f"max abs err {err.max():.3e} (lengths={lengths[:8]}..)"
    if raw.dtype == torch.bfloat16:
        # bf16 output = the fp32-output result (held to the strict bar by the callers that ask for it) rounded once
        _, raw32 = hp.gpu_attn(q, k, v, cu, ms, scale, torch.float32, extra_rows=3)
        assert torch.equal(raw[:T].view(torch.int16), raw32[:T].to(torch.bfloat16).view(torch.int16))
    return float(err.max()) if T else 0.0


@pytest.mark.parametrize("n", [1, 2, 3, 15, 16, 17, 31, 32, 33, 40, 47, 48, 49, 63, 64, 65, 100, 127, 128,
                               129, 191, 192, 193, 197, 255, 256, 257, 300, 577])
def test_single_sequence_lengths_fp16(n):
    check([n], 2, "f16", 100 + n)


@pytest.mark.parametrize("H", [1, 5, 7, 16])
def test_head_counts_and_several_dispatch_batches(H):
    """The (image, head) pair of a work-group comes from a multiply with a host-made reciprocal of H, and pairs
    beyond 512 go to further dispatch batches (the third grid dimension): head counts that are not the usual 12,
    with enough images for two or three batches."""
    B = 1100 // H + 3
    rng = np.random.default_rng(77 + H)
    lengths = [int(v) for v in rng.integers(0, 70, size=B)]
    lengths[0], lengths[-1] = 69, 1
    assert B * H > 1024
    check(lengths, H, "f16", 900 + H, max_seqlen=70)


def test_loose_bound_many_surplus_q_tiles():
    """A bound far above every length: 300 q-tiles in the second grid dimension, all but two of them without rows."""
    check([40, 3, 70, 0, 129], 2, "f16", 4343, max_seqlen=64 * 300)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_last_tile_takes_a_tail_of_up_to_16_keys_along(dtype):
    """Large launches (not the key-split form) run a last tile of 65..80 keys in one pass when at least two full
    tiles precede the tail: every length around the window's edges behind one, two and three full tiles, plus the
    64k+1 lengths of unpruned ViTs."""
    lengths = list(range(63, 84)) + list(range(127, 147)) + [191, 192, 193, 197, 207, 208, 209, 577]
    assert len(lengths) * 6 * 2 > 256                          # more 64-row q-tiles than the key-split form takes
    check(lengths, 6, dtype, 4242, max_seqlen=577)


@pytest.mark.parametrize("n", [1, 2, 17, 40, 64, 65, 197, 577])
@pytest.mark.parametrize("out", ["same", "f32"])
def test_single_sequence_lengths_bf16(n, out):
    check([n], 2, "bf16", 200 + n, out_dtype=torch.float32 if out == "f32" else None)


@pytest.mark.parametrize("n", [1, 40, 65, 197])
def test_fp16_in_fp32_out(n):
    check([n, 3, n], 3, "f16", 300 + n, out_dtype=torch.float32)


def test_tiny_workload():
    w = wl.tiny()
    q, k, v = w.qkv()
    cu = hp.cu_from_lengths(w.lengths)
    want = oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), cu, w.scale, "f16", threads=8)
    got, _ = hp.gpu_attn(q, k, v, cu, w.N, w.scale)
    assert np.max(np.abs(got - want)) <= TOL


@pytest.mark.parametrize("seed", range(6))
def test_ragged_batches_with_empty_and_single_token_images(seed):
    rng = np.random.default_rng(seed)
    lengths = [int(v) for v in rng.integers(0, 200, size=12)]
    lengths[rng.integers(12)] = 0
    lengths[rng.integers(12)] = 1
    lengths[0] = 0 if seed % 2 else lengths[0]
    lengths[-1] = 0 if seed % 3 == 0 else lengths[-1]
    check(lengths, 4, "f16" if seed % 2 == 0 else "bf16", 400 + seed, max_seqlen=199)


def test_all_images_empty():
    q, k, v = _qkv(4, 2, "f16", 1)
    got, raw = hp.gpu_attn(q[:0], k[:0], v[:0], hp.cu_from_lengths([0, 0, 0]), 197, 0.125, extra_rows=4)
    assert np.all(got == 77.0)


def test_headline_config_full_parity():
    """DeiT-B shape, B=32, 80 % pruned, with the launch arguments the benchmark uses
    (max_seqlen = N, no host knowledge of the lengths)."""
    w = wl.deit_b_pruned(0.2)
    q, k, v = w.qkv()
    cu = hp.cu_from_lengths(w.lengths)
    want = oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), cu, w.scale, "f16", threads=8)
    got, _ = hp.gpu_attn(q, k, v, cu, w.N, w.scale)
    err = np.abs(got - want)
    assert err.max() <= TOL
    assert err.mean() < 2e-4                                  # paper's kernel rows: mean 1.6e-5..3e-5 vs fp16 SDPA


@pytest.mark.parametrize("p", wl.SWEEP_KEEP_PROBS)
def test_sweep_bf16_fp32_out(p):
    w = wl.deit_b_pruned(p, 32, "bf16", 1002)
    q, k, v = w.qkv()
    cu = hp.cu_from_lengths(w.lengths)
    want = oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), cu, w.scale, "bf16", threads=8)
    got, raw32 = hp.gpu_attn(q, k, v, cu, w.N, w.scale, out_dtype=torch.float32)
    assert np.max(np.abs(got - want)) <= TOL
    got, raw16 = hp.gpu_attn(q, k, v, cu, w.N, w.scale)       # bf16 out: output rounding added
    assert np.all(np.abs(got - want) <= TOL + np.abs(want) * 2.0 ** -8)
    # the bf16-output path is the strictly checked fp32-output path plus ONE round-to-nearest-even
    assert torch.equal(raw16.view(torch.int16), raw32.to(torch.bfloat16).view(torch.int16))
    # where the output rounding is small next to the bar (|o| < 1/4: half an ulp <= 2^-11) the strict bar holds
    small = np.abs(want) < 0.25
    assert np.all(np.abs(got - want)[small] <= TOL)


@pytest.mark.parametrize("B", [1, 2, 4, 32])
def test_serving_384(B):
    w = wl.serving_384(B)
    q, k, v = w.qkv()
    cu = hp.cu_from_lengths(w.lengths)
    want = oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), cu, w.scale, "f16", threads=8)
    got, _ = hp.gpu_attn(q, k, v, cu, w.N, w.scale)
    assert np.max(np.abs(got - want)) <= TOL


def test_pipeline_layer1_sampled_rows():
    """B=64, every token kept (T = 12,608): the oracle checks sampled rows one by one."""
    w = wl.pipeline()[0]
    q, k, v = w.qkv()
    cu = hp.cu_from_lengths(w.lengths)
    got, _ = hp.gpu_attn(q, k, v, cu, w.N, w.scale)
    qw, kw, vw = wl.to_words(q), wl.to_words(k), wl.to_words(v)
    rng = np.random.default_rng(7)
    for _ in range(200):
        i, h = int(rng.integers(w.B)), int(rng.integers(w.H))
        r = int(rng.integers(cu[i + 1] - cu[i]))
        _, o = oracle.attn_row(qw, kw, vw, cu, i, h, r, w.scale, "f16")
        assert np.max(np.abs(got[cu[i] + r, h] - o)) <= TOL
    assert np.all(np.isfinite(got))


@pytest.mark.parametrize("scale", [0.0, -0.125, 1.0, 0.02])
def test_scales(scale):
    check([5, 70, 33], 2, "f16", 500, scale=scale, tol=TOL if abs(scale) < 1 else 4e-3)


def test_single_token_sequences_return_v_bits():
    lengths = [1] * 9
    q, k, v = _qkv(9, 3, "f16", 600)
    got, raw = hp.gpu_attn(q, k, v, hp.cu_from_lengths(lengths), 1, 0.125)
    assert torch.equal(raw.view(torch.int16), v.view(torch.int16))


def test_identical_v_rows_are_returned_within_one_ulp():
    n, H = 50, 2
    q, k, _ = _qkv(n, H, "f16", 601)
    v1 = torch.randn(1, H, 64, generator=torch.Generator().manual_seed(3)).to(torch.float16)
    v = v1.repeat(n, 1, 1).contiguous()
    got, raw = hp.gpu_attn(q, k, v, hp.cu_from_lengths([n]), n, 0.125)
    ulp = np.maximum(np.abs(v1.to(torch.float64).numpy()), 2.0 ** -14) * 2.0 ** -10
    assert np.all(np.abs(got - v1.to(torch.float64).numpy()) <= ulp)


def test_ragged_isolation_bit_exact():
    """Replacing every token of image 1 must leave the other images' output bits unchanged: keys of
    a neighbouring image never leak into a tile tail."""
    lengths = [40, 70, 23, 197]
    cu = hp.cu_from_lengths(lengths)
    q, k, v = _qkv(int(cu[-1]), 3, "f16", 602)
    q2, k2, v2 = _qkv(int(cu[-1]), 3, "f16", 603)
    for a, b in ((q, q2), (k, k2), (v, v2)):
        b[:40] = a[:40]
        b[110:] = a[110:]
    _, r1 = hp.gpu_attn(q, k, v, cu, 197, 0.125)
    _, r2 = hp.gpu_attn(q2, k2, v2, cu, 197, 0.125)
    a, b = r1.view(torch.int16), r2.view(torch.int16)
    assert torch.equal(a[:40], b[:40]) and torch.equal(a[110:], b[110:])
    assert not torch.equal(a[40:110], b[40:110])


def test_run_to_run_determinism():
    w = wl.deit_b_pruned(0.4, B=8)
    q, k, v = w.qkv()
    cu = hp.cu_from_lengths(w.lengths)
    _, r1 = hp.gpu_attn(q, k, v, cu, w.N, w.scale)
    for _ in range(3):
        _, r2 = hp.gpu_attn(q, k, v, cu, w.N, w.scale)
        assert torch.equal(r1.view(torch.int16), r2.view(torch.int16))


def test_max_seqlen_only_bounds_the_grid():
    """Any bound >= max n gives the same bits."""
    lengths = [30, 64, 10]
    cu = hp.cu_from_lengths(lengths)
    q, k, v = _qkv(int(cu[-1]), 2, "f16", 604)
    _, a = hp.gpu_attn(q, k, v, cu, 64, 0.125)
    _, b = hp.gpu_attn(q, k, v, cu, 1000, 0.125)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def _checked(lengths, bound, H=2, seed=606):
    """ragged_attn_checked on sentinel-filled output; returns (raw output, flags word, inputs)."""
    from paper_2604_15408_amd import binding
    cu = hp.cu_from_lengths(lengths)
    q, k, v = _qkv(int(cu[-1]), H, "f16", seed)
    dev = "cuda:0"
    o = torch.full(q.shape, 77.0, dtype=q.dtype, device=dev)
    flags = torch.zeros(1, dtype=torch.int32, device=dev)
    binding.ragged_attn_checked(q.to(dev), k.to(dev), v.to(dev), o, torch.from_numpy(cu).to(dev), bound, 0.125, flags)
    torch.cuda.synchronize()
    return o.cpu(), int(flags.item()), (q, k, v, cu)


def _oracle_rows(q, k, v, cu):
    return oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), cu, 0.125, "f16", threads=8)


def test_checked_attention_reports_a_bound_that_is_too_small():
    """max_seqlen below some n_i: the flag bit is set on the device, every kernel exits normally, every row at a
    position below the bound is computed (oracle bar), rows of the offending image at or past the bound rounded
    up to the 64-row tile stay untouched, and the other images are complete."""
    from paper_2604_15408_amd import binding
    lengths = [30, 150, 10, 64]
    raw, flags, (q, k, v, cu) = _checked(lengths, bound=64)         # image 1 has 150 > 64 tokens
    assert flags & binding.FLAG_SEQLEN_EXCEEDED
    want = _oracle_rows(q, k, v, cu)
    got = raw.to(torch.float64).numpy()
    covered = np.ones(int(cu[-1]), dtype=bool)
    covered[cu[1] + 64: cu[2]] = False                               # query rows 64.. of image 1 are lost
    assert np.max(np.abs(got[covered] - want[covered])) <= TOL
    assert bool((raw[~covered] == 77.0).all())
    # the same call without the flag word gives the same bits
    _, plain = hp.gpu_attn(q, k, v, cu, 64, 0.125)
    assert torch.equal(raw.view(torch.int16), plain.view(torch.int16))


def test_checked_attention_keeps_the_flag_clear_when_the_bound_holds():
    lengths = [30, 150, 10, 64]
    for bound in (150, 197, 1000):
        raw, flags, (q, k, v, cu) = _checked(lengths, bound=bound)
        assert flags == 0
        _, full = hp.gpu_attn(q, k, v, cu, bound, 0.125)
        assert torch.equal(raw.view(torch.int16), full.view(torch.int16))
        assert np.max(np.abs(raw.to(torch.float64).numpy() - _oracle_rows(q, k, v, cu))) <= TOL
    # a bound just below n_i is reported too; rows below the bound are all there, rows at or past it may be missing
    raw, flags, (q, k, v, cu) = _checked(lengths, bound=140)
    assert flags == 1
    want = _oracle_rows(q, k, v, cu)
    got = raw.to(torch.float64).numpy()
    below = np.ones(int(cu[-1]), dtype=bool)
    below[cu[1] + 140: cu[2]] = False
    assert np.max(np.abs(got[below] - want[below])) <= TOL
    tail = raw[cu[1] + 140: cu[2]]
    for row, ref in zip(tail.to(torch.float64).numpy(), want[cu[1] + 140: cu[2]]):
        assert bool((row == 77.0).all()) or np.max(np.abs(row - ref)) <= TOL      # untouched, or computed whole


def test_small_launches_split_the_keys_over_the_wavefronts():
    """Launches of few work-groups take the key-split form (16-query work-groups, partial results merged through
    LDS); large ones the 64-query form.  The same sequences through both: each within the oracle bar, single-tile
    sequences bit-identical (nothing to merge), longer ones equal within rounding."""
    lengths = [30, 150, 10, 64, 197, 1, 65, 256, 257, 300]
    cu = hp.cu_from_lengths(lengths)
    q, k, v = _qkv(int(cu[-1]), 2, "f16", 611)
    want = _oracle_rows(q, k, v, cu)
    small, raw_small = hp.gpu_attn(q, k, v, cu, 300, 0.125)          # 20 pairs x 5 q-tiles: key-split form
    # the same rows inside a batch large enough for the 64-query form: 60 images, 120 pairs x 5 q-tiles
    reps = 6
    cu_big = hp.cu_from_lengths(lengths * reps)
    qb, kb, vb = (t.repeat(reps, 1, 1).contiguous() for t in (q, k, v))
    big, raw_big = hp.gpu_attn(qb, kb, vb, cu_big, 300, 0.125)
    T = int(cu[-1])
    assert np.max(np.abs(small - want)) <= TOL and np.max(np.abs(big[:T] - want)) <= TOL
    for r in range(1, reps):                                        # copies of a sequence inside one launch: same bits
        assert torch.equal(raw_big[:T].view(torch.int16), raw_big[r * T:(r + 1) * T].view(torch.int16))
    a, b = raw_small.view(torch.int16), raw_big[:T].view(torch.int16)
    for i, n in enumerate(lengths):
        rows = slice(int(cu[i]), int(cu[i + 1]))
        if n <= 64:
            assert torch.equal(a[rows], b[rows])
        else:
            assert np.max(np.abs(small[rows] - big[rows])) <= 1e-3


def test_permutation_equivariance_within_tolerance():
    n = 90
    cu = hp.cu_from_lengths([n])
    q, k, v = _qkv(n, 2, "f16", 605)
    perm = torch.randperm(n, generator=torch.Generator().manual_seed(2))
    a, _ = hp.gpu_attn(q, k, v, cu, n, 0.125)
    b, _ = hp.gpu_attn(q[perm].contiguous(), k[perm].contiguous(), v[perm].contiguous(), cu, n, 0.125)
    assert np.max(np.abs(a[perm.numpy()] - b)) <= TOL
