"""Pins for the CPU oracle's pack / unpack (CPU only): NumPy boolean indexing, cumsum and
flatnonzero are the library routines these reduce to (paper Section 4.1); plus the round-trip
identities and the closed form of the tiny configuration."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import workloads as wl


def _case(B, N, C, p, seed):
    keep = wl.keep_bernoulli(B, N, p, seed).numpy()
    rng = np.random.default_rng(seed)
    x = rng.integers(0, 65536, (B, N, C), dtype=np.uint16)
    return x, keep


@pytest.mark.parametrize("B,N,C,p,seed", [(1, 1, 8, 1.0, 0), (3, 17, 8, 0.5, 1), (4, 197, 24, 0.2, 2),
                                          (2, 64, 16, 0.0, 3), (5, 33, 8, 1.0, 4)])
def test_pack_equals_numpy_boolean_indexing(B, N, C, p, seed):
    x, keep = _case(B, N, C, p, seed)
    packed, cu, gidx = oracle.pack(x, keep)
    assert np.array_equal(packed, x[keep.astype(bool)])
    assert np.array_equal(cu, np.concatenate([[0], np.cumsum(keep.sum(axis=1))]))
    assert np.array_equal(gidx, np.flatnonzero(keep.reshape(-1)))
    assert cu.dtype == np.int32 and gidx.dtype == np.int32


def test_any_nonzero_byte_counts_as_keep():
    x, keep = _case(2, 9, 8, 0.5, 5)
    loud = keep * np.array([1, 2, 255, 7, 128, 1, 64, 3, 9], dtype=np.uint8)
    a = oracle.pack(x, keep)
    b = oracle.pack(x, loud)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)


def test_tiny_configuration_closed_form():
    w = wl.tiny()
    assert w.lengths == [197, 40]
    x = wl.to_words(w.features())
    packed, cu, gidx = oracle.pack(x, w.keep.numpy())
    assert cu.tolist() == [0, 197, 237]
    assert packed.shape == (237, 192)
    assert np.array_equal(gidx[:197], np.arange(197))
    assert gidx[197] == 197                              # CLS of image 1 leads its packed sequence
    assert np.array_equal(packed[197], x[1, 0])


def test_all_dropped_image_and_all_dropped_batch():
    x, _ = _case(3, 5, 8, 0.5, 6)
    keep = np.zeros((3, 5), dtype=np.uint8)
    keep[1, [0, 3]] = 1
    packed, cu, gidx = oracle.pack(x, keep)
    assert cu.tolist() == [0, 0, 2, 2] and gidx.tolist() == [5, 8]
    packed, cu, gidx = oracle.pack(x, np.zeros((3, 5), dtype=np.uint8))
    assert packed.shape == (0, 8) and cu.tolist() == [0, 0, 0, 0] and gidx.size == 0


@pytest.mark.parametrize("fill_mode", [0, 1])
def test_unpack_equals_numpy_scatter(fill_mode):
    x, keep = _case(4, 23, 8, 0.4, 7)
    packed, cu, _ = oracle.pack(x, keep)
    sentinel = np.full_like(x, 0xBEEF)
    out = oracle.unpack(packed, keep, cu, 8, fill_mode, out_init=sentinel)
    want = sentinel.copy() if fill_mode == 0 else np.zeros_like(x)
    want[keep.astype(bool)] = packed
    assert np.array_equal(out, want)


def test_unpack_after_pack_is_identity_on_kept_tokens_and_pack_after_unpack_is_identity():
    x, keep = _case(3, 31, 16, 0.3, 8)
    packed, cu, gidx = oracle.pack(x, keep)
    out = oracle.unpack(packed, keep, cu, 16, 1)
    kb = keep.astype(bool)
    assert np.array_equal(out[kb], x[kb])
    assert not out[~kb].any()
    repacked, cu2, gidx2 = oracle.pack(out, keep)
    assert np.array_equal(repacked, packed) and np.array_equal(cu2, cu) and np.array_equal(gidx2, gidx)


def test_unpack_distinguishes_rows():
    """Rows carry their own index, so an off-by-one rank or a wrong cu_seqlens offset shows."""
    keep = np.array([[1, 0, 1, 1], [0, 1, 0, 1]], dtype=np.uint8)
    cu = np.array([0, 3, 5], dtype=np.int32)
    src = (np.arange(5, dtype=np.uint16)[:, None] + 100) * np.ones((1, 8), dtype=np.uint16)
    out = oracle.unpack(src, keep, cu, 8, 1)
    assert out[:, :, 0].tolist() == [[100, 0, 101, 102], [0, 103, 0, 104]]


def test_workload_generators_are_seeded_and_shaped():
    a, b = wl.deit_b_pruned(0.2), wl.deit_b_pruned(0.2)
    assert torch.equal(a.keep, b.keep) and torch.equal(a.features(), b.features())
    assert a.keep.shape == (32, 197) and bool(a.keep[:, 0].all())
    assert 1000 < a.T < 1600                              # E[T] = 32 * (1 + 196*0.2) = 1286
    s = wl.serving_384(4)
    assert s.keep.shape == (4, 577) and bool(s.keep[:, 0].all())
    masks = wl.pipeline_masks()
    assert len(masks) == 12 and int(masks[0].sum()) == 64 * 197
    assert all(int((masks[l + 1] > masks[l]).sum()) == 0 for l in range(11))   # tokens never return
    assert int(masks[2].sum()) < int(masks[1].sum()) and bool(masks[-1][:, 0].all())
    assert [w.dtype for w in wl.sweep()] == ["bf16"] * 6
    assert wl.sweep()[0].T == 32 * 197


# ---- staying packed: re-pack and CLS extraction ---------------------------------------------------

def test_repack_equals_numpy_indexing_and_boundary_counts():
    x, keep = _case(5, 29, 8, 0.6, 20)
    keep[2, :] = 0                                            # an empty image in the middle
    packed, cu, _ = oracle.pack(x, keep)
    T = packed.shape[0]
    rows = (np.random.default_rng(3).random(T + 5) < 0.5).astype(np.uint8)   # extra bytes past T are ignored
    out, cu2, g2 = oracle.repack(packed, rows, cu)
    sel = rows[:T].astype(bool)
    assert np.array_equal(out, packed[sel])
    assert np.array_equal(g2, np.flatnonzero(sel))
    csum = np.concatenate([[0], np.cumsum(sel)])
    assert np.array_equal(cu2, csum[cu])


def test_repack_of_pack_equals_pack_with_both_masks():
    """Pruning an already packed buffer must give what packing with the combined mask gives."""
    x, keep1 = _case(4, 41, 16, 0.7, 21)
    keep2 = wl.keep_bernoulli(4, 41, 0.5, 22).numpy()
    packed1, cu1, _ = oracle.pack(x, keep1)
    rows = keep2[keep1.astype(bool)]                           # second decision, per surviving token
    out, cu2, g2 = oracle.repack(packed1, rows, cu1)
    want_packed, want_cu, want_gidx = oracle.pack(x, keep1 & keep2)
    assert np.array_equal(out, want_packed) and np.array_equal(cu2, want_cu)
    _, _, gidx1 = oracle.pack(x, keep1)
    assert np.array_equal(gidx1[g2], want_gidx)                # composing the two gather maps


def test_repack_keep_all_and_keep_none():
    x, keep = _case(3, 17, 8, 0.5, 23)
    packed, cu, _ = oracle.pack(x, keep)
    T = packed.shape[0]
    out, cu2, g2 = oracle.repack(packed, np.ones(T, np.uint8), cu)
    assert np.array_equal(out, packed) and np.array_equal(cu2, cu) and np.array_equal(g2, np.arange(T))
    out, cu2, g2 = oracle.repack(packed, np.zeros(T, np.uint8), cu)
    assert out.shape == (0, 8) and not cu2.any() and g2.size == 0


def test_cls_extract_is_first_row_of_each_image():
    x, keep = _case(5, 23, 8, 0.4, 24)
    keep[:, 0] = 1
    keep[3, :] = 0                                            # image 3 has no rows at all
    packed, cu, _ = oracle.pack(x, keep)
    cls = oracle.cls_extract(packed, cu)
    for i in range(5):
        if i == 3:
            assert not cls[i].any()
        else:
            assert np.array_equal(cls[i], x[i, 0])             # CLS is token 0 and always kept
