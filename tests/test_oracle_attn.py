"""Pins for the CPU oracle's attention (CPU only).

The oracle is the plain definition of per-image bidirectional attention (paper Section 4.2).  It is
pinned here against things that are NOT the oracle: an independently written padded+masked NumPy
attention (the paper's own equivalence claim, Section 5.6 "Numerical Equivalence"), torch's
float64 scaled_dot_product_attention, closed forms, and invariants that a dropped term, a wrong
index, a swapped operand or a forgotten scale would break.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import workloads as wl


def _rand_words(shape, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    t = torch.randn(*shape, generator=g, dtype=torch.float32)
    t = t.to(torch.float16 if dtype == "f16" else torch.bfloat16)
    return wl.to_words(t), t.to(torch.float64).numpy()


def _cu(lengths):
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


def padded_masked_attention(qf, kf, vf, keep, scale):
    """Independent checker: scatter the packed rows back to [B,N,H,D], run dense attention with the
    scores of dropped keys set to -inf, then gather the kept query rows (NumPy, float64)."""
    B, N = keep.shape
    T, H, D = qf.shape
    flat = np.flatnonzero(keep.reshape(-1))
    assert flat.size == T
    Qp = np.zeros((B * N, H, D)); Kp = np.zeros((B * N, H, D)); Vp = np.zeros((B * N, H, D))
    Qp[flat], Kp[flat], Vp[flat] = qf, kf, vf
    Qp, Kp, Vp = (a.reshape(B, N, H, D).transpose(0, 2, 1, 3) for a in (Qp, Kp, Vp))
    S = np.einsum("bhqd,bhkd->bhqk", Qp, Kp) * scale
    S = np.where(keep[:, None, None, :].astype(bool), S, -np.inf)
    S = S - S.max(axis=-1, keepdims=True)
    P = np.exp(S)
    P = P / P.sum(axis=-1, keepdims=True)
    O = np.einsum("bhqk,bhkd->bhqd", P, Vp).transpose(0, 2, 1, 3).reshape(B * N, H, D)
    return O[flat]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_decoders_exhaustive(dtype):
    words = np.arange(65536, dtype=np.uint16)
    got = oracle.decode(words, dtype)
    if dtype == "f16":
        want = words.view(np.float16).astype(np.float64)
    else:
        want = torch.from_numpy(words.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_matches_padded_masked_bruteforce(dtype, seed):
    B, N, H, D = 3, 11, 2, 8
    keep = wl.keep_bernoulli(B, N, 0.5, seed + 50).numpy()
    T = int(keep.sum())
    qw, qf = _rand_words((T, H, D), dtype, seed * 3 + 1)
    kw, kf = _rand_words((T, H, D), dtype, seed * 3 + 2)
    vw, vf = _rand_words((T, H, D), dtype, seed * 3 + 3)
    cu = _cu(keep.sum(axis=1))
    scale = 0.37
    got = oracle.attn(qw, kw, vw, cu, scale, dtype)
    want = padded_masked_attention(qf, kf, vf, keep, float(np.float32(scale)))
    assert np.max(np.abs(got - want)) < 1e-13


def test_matches_padded_masked_at_tiny_workload_shape():
    w = wl.tiny()
    keep = w.keep.numpy()
    q, k, v = w.qkv()
    cu = _cu(w.lengths)
    got = oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), cu, w.scale, "f16", threads=4)
    want = padded_masked_attention(*(t.to(torch.float64).numpy() for t in (q, k, v)), keep, w.scale)
    assert got.shape == (237, 3, 64)
    assert np.max(np.abs(got - want)) < 1e-13


@pytest.mark.parametrize("n,D,scale", [(1, 64, 0.125), (7, 64, 0.125), (40, 64, 0.125), (33, 32, 0.3)])
def test_single_sequence_matches_torch_sdpa_float64(n, D, scale):
    H = 3
    qw, qf = _rand_words((n, H, D), "f16", 11)
    kw, kf = _rand_words((n, H, D), "f16", 12)
    vw, vf = _rand_words((n, H, D), "f16", 13)
    got = oracle.attn(qw, kw, vw, _cu([n]), scale, "f16")
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2).unsqueeze(0) for a in (qf, kf, vf))
    want = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, scale=float(np.float32(scale)))[0].permute(1, 0, 2).numpy()
    assert np.max(np.abs(got - want)) < 1e-13


def test_threads_do_not_change_bits():
    lengths = [5, 0, 9, 1, 17]
    T = sum(lengths)
    qw, _ = _rand_words((T, 4, 16), "f16", 1)
    kw, _ = _rand_words((T, 4, 16), "f16", 2)
    vw, _ = _rand_words((T, 4, 16), "f16", 3)
    a = oracle.attn(qw, kw, vw, _cu(lengths), 0.25, "f16", threads=1)
    b = oracle.attn(qw, kw, vw, _cu(lengths), 0.25, "f16", threads=5)
    assert np.array_equal(a, b)


def test_single_token_sequence_returns_its_v_row_exactly():
    lengths = [1, 3, 1]
    T = sum(lengths)
    qw, _ = _rand_words((T, 2, 8), "f16", 4)
    kw, _ = _rand_words((T, 2, 8), "f16", 5)
    vw, vf = _rand_words((T, 2, 8), "f16", 6)
    out = oracle.attn(qw, kw, vw, _cu(lengths), 0.125, "f16")
    assert np.array_equal(out[0], vf[0])
    assert np.array_equal(out[4], vf[4])


def test_scale_zero_gives_mean_of_v_per_image():
    lengths = [4, 6]
    T = sum(lengths)
    qw, _ = _rand_words((T, 2, 8), "bf16", 7)
    kw, _ = _rand_words((T, 2, 8), "bf16", 8)
    vw, vf = _rand_words((T, 2, 8), "bf16", 9)
    out = oracle.attn(qw, kw, vw, _cu(lengths), 0.0, "bf16")
    for s, e in [(0, 4), (4, 10)]:
        mean = vf[s:e].mean(axis=0)
        for r in range(s, e):
            assert np.max(np.abs(out[r] - mean)) < 1e-15


def test_identical_v_rows_are_returned_unchanged():
    n, H, D = 9, 2, 8
    qw, _ = _rand_words((n, H, D), "f16", 10)
    kw, _ = _rand_words((n, H, D), "f16", 11)
    v1w, v1f = _rand_words((1, H, D), "f16", 12)
    vw = np.repeat(v1w, n, axis=0)
    out = oracle.attn(qw, kw, vw, _cu([n]), 0.125, "f16")
    assert np.max(np.abs(out - v1f)) < 1e-15


def test_two_token_closed_form():
    """q=(1,0), k0=(0,0), k1=(1,0), scale 1: scores (0,1) so p1 = e/(1+e) for query 0; query 1 is
    q=(2,0): scores (0,2).  Output = v0 + p1 (v1 - v0).  A swapped Q/K or V index changes it."""
    f = lambda rows: np.array(rows, dtype=np.float16).reshape(2, 1, 2).view(np.uint16)
    q = f([[1, 0], [2, 0]]); k = f([[0, 0], [1, 0]]); v = f([[1, -2], [3, 4]])
    out = oracle.attn(q, k, v, _cu([2]), 1.0, "f16")
    for r, s in [(0, 1.0), (1, 2.0)]:
        p1 = math.exp(s) / (1.0 + math.exp(s))
        want = np.array([1 + p1 * 2, -2 + p1 * 6])
        assert np.max(np.abs(out[r, 0] - want)) < 1e-15


def test_scale_is_applied_to_the_dot_product():
    """Same as above with scale 0.5 on doubled keys must agree with scale 1 (catches a dropped or
    squared scale)."""
    f = lambda rows: np.array(rows, dtype=np.float16).reshape(2, 1, 2).view(np.uint16)
    q = f([[1, 0], [2, 0]]); v = f([[1, -2], [3, 4]])
    a = oracle.attn(q, f([[0, 0], [1, 0]]), v, _cu([2]), 1.0, "f16")
    b = oracle.attn(q, f([[0, 0], [2, 0]]), v, _cu([2]), 0.5, "f16")
    assert np.max(np.abs(a - b)) < 1e-15


def test_large_scale_selects_the_argmax_key():
    n, H, D = 12, 2, 8
    qw, qf = _rand_words((n, H, D), "f16", 20)
    kw, kf = _rand_words((n, H, D), "f16", 21)
    vw, vf = _rand_words((n, H, D), "f16", 22)
    out = oracle.attn(qw, kw, vw, _cu([n]), 4096.0, "f16")
    for h in range(H):
        S = qf[:, h] @ kf[:, h].T
        top2 = np.sort(S, axis=1)[:, -2:]
        assert np.all(top2[:, 1] - top2[:, 0] > 1e-2)          # unique maxima on these inputs
        assert np.max(np.abs(out[:, h] - vf[np.argmax(S, axis=1), h])) < 1e-12


def test_probabilities_sum_to_one_and_reproduce_the_row():
    lengths = [6, 13]
    T = sum(lengths)
    qw, _ = _rand_words((T, 2, 16), "f16", 30)
    kw, _ = _rand_words((T, 2, 16), "f16", 31)
    vw, vf = _rand_words((T, 2, 16), "f16", 32)
    cu = _cu(lengths)
    full = oracle.attn(qw, kw, vw, cu, 0.25, "f16")
    for i, h, r in [(0, 0, 0), (0, 1, 5), (1, 0, 12), (1, 1, 3)]:
        p, o = oracle.attn_row(qw, kw, vw, cu, i, h, r, 0.25, "f16")
        assert p.shape == (lengths[i],) and np.all(p > 0)
        assert abs(p.sum() - 1.0) < 1e-14
        assert np.array_equal(o, full[cu[i] + r, h])
        assert np.max(np.abs(p @ vf[cu[i]:cu[i + 1], h] - o)) < 1e-14


def test_adding_a_vector_to_every_key_changes_nothing():
    """Scores of a row all shift by q.u, which softmax ignores.  Integer-valued inputs keep the
    shifted keys exact in fp16."""
    rng = np.random.default_rng(5)
    n, H, D = 10, 2, 8
    mk = lambda a: a.astype(np.float16).view(np.uint16)
    q = rng.integers(-3, 4, (n, H, D)); k = rng.integers(-3, 4, (n, H, D))
    v = rng.integers(-3, 4, (n, H, D)); u = rng.integers(-2, 3, (1, H, D))
    a = oracle.attn(mk(q), mk(k), mk(v), _cu([n]), 0.125, "f16")
    b = oracle.attn(mk(q), mk(k + u), mk(v), _cu([n]), 0.125, "f16")
    assert np.max(np.abs(a - b)) < 1e-13


def test_permuting_a_sequence_permutes_its_output():
    lengths = [7, 9]
    T = sum(lengths)
    qw, _ = _rand_words((T, 2, 8), "f16", 40)
    kw, _ = _rand_words((T, 2, 8), "f16", 41)
    vw, _ = _rand_words((T, 2, 8), "f16", 42)
    cu = _cu(lengths)
    perm = np.arange(T)
    perm[7:] = 7 + np.random.default_rng(3).permutation(9)
    a = oracle.attn(qw, kw, vw, cu, 0.2, "f16")
    b = oracle.attn(qw[perm], kw[perm], vw[perm], cu, 0.2, "f16")
    assert np.array_equal(a[:7], b[:7])
    assert np.max(np.abs(a[perm] - b)) < 1e-14


def test_ragged_isolation():
    """Changing every token of image 1 leaves images 0 and 2 bit-identical: no key of a
    neighbouring image leaks into a sequence (Alg. 1 loads whole tiles without a bound)."""
    lengths = [5, 8, 3]
    T = sum(lengths)
    qw, _ = _rand_words((T, 2, 8), "f16", 50)
    kw, _ = _rand_words((T, 2, 8), "f16", 51)
    vw, _ = _rand_words((T, 2, 8), "f16", 52)
    q2, k2, v2 = qw.copy(), kw.copy(), vw.copy()
    junk, _ = _rand_words((8, 2, 8), "f16", 53)
    q2[5:13], k2[5:13], v2[5:13] = junk, junk[::-1], junk
    cu = _cu(lengths)
    a = oracle.attn(qw, kw, vw, cu, 0.3, "f16")
    b = oracle.attn(q2, k2, v2, cu, 0.3, "f16")
    assert np.array_equal(a[:5], b[:5]) and np.array_equal(a[13:], b[13:])
    assert not np.array_equal(a[5:13], b[5:13])


def test_output_lies_in_the_convex_hull_of_v():
    lengths = [4, 20]
    T = sum(lengths)
    qw, _ = _rand_words((T, 3, 8), "bf16", 60)
    kw, _ = _rand_words((T, 3, 8), "bf16", 61)
    vw, vf = _rand_words((T, 3, 8), "bf16", 62)
    cu = _cu(lengths)
    out = oracle.attn(qw, kw, vw, cu, 0.35, "bf16")
    for i in range(2):
        s, e = cu[i], cu[i + 1]
        lo, hi = vf[s:e].min(axis=0), vf[s:e].max(axis=0)
        assert np.all(out[s:e] >= lo - 1e-14) and np.all(out[s:e] <= hi + 1e-14)


def test_empty_sequences_and_empty_batch():
    qw, _ = _rand_words((3, 2, 8), "f16", 70)
    out = oracle.attn(qw, qw, qw, _cu([0, 3, 0]), 0.125, "f16")
    assert out.shape == (3, 2, 8) and np.all(np.isfinite(out))
    empty = np.zeros((0, 2, 8), dtype=np.uint16)
    assert oracle.attn(empty, empty, empty, _cu([0, 0]), 0.125, "f16").shape == (0, 2, 8)


def test_fp16_rounding_of_the_oracle_is_within_the_papers_error_band():
    """The paper reports kernel max|delta| of 4.88e-4 .. 9.77e-4 between two fp16 implementations
    (Section 5.6, numerical-equivalence table; values stored in tests/golden).  Rounding the fp64
    oracle to fp16 must land in the same band on N(0,1) inputs -- an order-of-magnitude check that
    the oracle's outputs are on the scale the paper measured."""
    import json, os
    golden = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_kernel_max_abs_diff.json")))
    w = wl.deit_b_pruned(0.2, B=4)
    q, k, v = w.qkv()
    out = oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), _cu(w.lengths), w.scale, "f16", threads=4)
    err = np.max(np.abs(out.astype(np.float16).astype(np.float64) - out))
    assert err <= 2 * max(golden["max_abs_diff"].values())
    assert err >= 0.1 * min(golden["max_abs_diff"].values())


# ---- attention on the padded layout (pack and unpack folded into the attention) -----------------

def _padded_case(B, N, H, D, p, dtype, seed):
    keep = wl.keep_bernoulli(B, N, p, seed).numpy()
    qw, qf = _rand_words((B, N, H, D), dtype, seed + 1)
    kw, kf = _rand_words((B, N, H, D), dtype, seed + 2)
    vw, vf = _rand_words((B, N, H, D), dtype, seed + 3)
    return keep, (qw, kw, vw), (qf, kf, vf)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_padded_attention_equals_pack_attend_unpack(dtype):
    """The folded variant must equal the composition of the three pinned stages."""
    B, N, H, D = 3, 13, 2, 8
    keep, (qw, kw, vw), _ = _padded_case(B, N, H, D, 0.5, dtype, 90)
    keep[1, :] = 0                                             # an image with nothing kept
    got = oracle.attn_padded(qw, kw, vw, keep, 0.3, dtype)
    kb = keep.astype(bool)
    cu = _cu(keep.sum(axis=1))
    packed = oracle.attn(qw[kb], kw[kb], vw[kb], cu, 0.3, dtype)
    want = np.zeros((B, N, H, D))
    want[kb] = packed
    assert np.array_equal(got, want)


def test_padded_attention_matches_masked_dense_numpy():
    B, N, H, D = 2, 9, 3, 4
    keep, (qw, kw, vw), (qf, kf, vf) = _padded_case(B, N, H, D, 0.6, "f16", 91)
    got = oracle.attn_padded(qw, kw, vw, keep, 0.25, "f16")
    S = np.einsum("bqhd,bkhd->bhqk", qf, kf) * 0.25
    S = np.where(keep[:, None, None, :].astype(bool), S, -np.inf)
    P = np.exp(S - S.max(axis=-1, keepdims=True))
    P /= P.sum(axis=-1, keepdims=True)
    O = np.einsum("bhqk,bkhd->bqhd", P, vf)
    kb = keep.astype(bool)
    assert np.max(np.abs(got[kb] - O[kb])) < 1e-13
    assert not got[~kb].any() and np.all(np.isfinite(got))


def test_padded_attention_ignores_dropped_tokens_entirely():
    """Garbage (even NaN patterns) in dropped rows of q, k, v must not reach any output."""
    B, N, H, D = 2, 10, 2, 4
    keep, (qw, kw, vw), _ = _padded_case(B, N, H, D, 0.5, "f16", 92)
    a = oracle.attn_padded(qw, kw, vw, keep, 0.5, "f16")
    kb = keep.astype(bool)
    q2, k2, v2 = qw.copy(), kw.copy(), vw.copy()
    for arr in (q2, k2, v2):
        arr[~kb] = 0x7E00                                      # fp16 NaN
    b = oracle.attn_padded(q2, k2, v2, keep, 0.5, "f16")
    assert np.array_equal(a, b)
