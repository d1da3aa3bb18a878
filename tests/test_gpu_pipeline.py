"""The whole pipeline inside HIP graphs: every entry point must be capturable (no allocation, no
synchronisation, no host read), and replays must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_15408_amd import workloads as wl
from paper_2604_15408_amd.harness import Path, Pipeline, StayPackedPipeline, capture
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _small_pipeline(B=6):
    masks = wl.pipeline_masks(B=B, seed=77)
    return [wl.Workload(f"pipe{l}", B, 197, 12, 64, "f16", 500 + l, m) for l, m in enumerate(masks)]


def test_single_step_graph_replays_match_eager():
    w = wl.deit_b_pruned(0.3, B=8)
    p = Path(w, fill_mode=1)
    p.step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (p.packed, p.cu, p.gidx, p.o, p.out)]
    g = capture(torch, p.step)
    for rep in range(4):
        for t in (p.packed, p.o, p.out):
            t.fill_(-3.0)                                   # eager work between the replays
        p.cu.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        T = int(p.cu[-1])
        assert T == w.T
        assert torch.equal(p.cu, want[1])
        assert torch.equal(p.gidx[:T], want[2][:T])
        assert torch.equal(p.packed[:T].view(torch.int16), want[0][:T].view(torch.int16))
        assert torch.equal(p.o[:T].view(torch.int16), want[3][:T].view(torch.int16))
        assert torch.equal(p.out.view(torch.int16), want[4].view(torch.int16))


def test_twelve_layer_loop_in_one_graph_matches_eager_and_oracle():
    layers = _small_pipeline()
    pipe = Pipeline(layers, fill_mode=1)
    pipe.run()
    torch.cuda.synchronize()
    eager_final = pipe.x[-1].clone()
    eager_cu = [c.clone() for c in pipe.cu]
    eager_o = [o.clone() for o in pipe.o]

    g = capture(torch, pipe.run)
    for rep in range(3):
        for t in pipe.x[1:]:
            t.fill_(9.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(pipe.x[-1].view(torch.int16), eager_final.view(torch.int16))
        for l in range(12):
            assert torch.equal(pipe.cu[l], eager_cu[l])
            assert torch.equal(pipe.o[l].view(torch.int16), eager_o[l].view(torch.int16))

    # oracle: lengths of every layer, attention of the last (most pruned) layer, final unpack
    for l, w in enumerate(layers):
        assert pipe.cu[l].cpu().numpy().tolist() == hp.cu_from_lengths(w.lengths).tolist()
    w = layers[-1]
    q, k, v = w.qkv()
    cu = hp.cu_from_lengths(w.lengths)
    want_o = oracle.attn(wl.to_words(q), wl.to_words(k), wl.to_words(v), cu, w.scale, "f16", threads=8)
    got_o = pipe.o[-1][: w.T].cpu().to(torch.float64).numpy()
    assert np.max(np.abs(got_o - want_o)) <= 2e-3
    want_x = oracle.unpack(wl.to_words(pipe.o[-1][: w.T].cpu()).reshape(w.T, w.C), w.keep.numpy(), cu, w.C, 1)
    assert np.array_equal(wl.to_words(pipe.x[-1].cpu()), want_x)
    # tokens dropped at an earlier layer stay dropped: their rows are zero after the last unpack
    assert not pipe.x[-1][~w.keep.bool().to("cuda:0")].any()


def test_full_size_twelve_layer_graph_against_the_oracle():
    """The 12-layer configuration at its full size (B = 64, N = 197, C = 768), one replay of the one-graph loop:
    cu_seqlens of every layer exactly, sampled attention rows of layers 3, 6, 9 and 12 (the layers that prune, and
    the last) against the oracle one row at a time, and the final unpack bit for bit."""
    layers = wl.pipeline()
    assert layers[0].B == 64 and len(layers) == 12
    pipe = Pipeline(layers, fill_mode=1)
    pipe.run()                                              # warms the code path; capture() runs it once more
    g = capture(torch, pipe.run)
    for t in pipe.x[1:] + pipe.o:
        t.fill_(9.0)
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    for l, w in enumerate(layers):
        assert pipe.cu[l].cpu().numpy().tolist() == hp.cu_from_lengths(w.lengths).tolist()
    rng = np.random.default_rng(11)
    for l in (2, 5, 8, 11):
        w = layers[l]
        q, k, v = (wl.to_words(t) for t in w.qkv())
        cu = hp.cu_from_lengths(w.lengths)
        got = pipe.o[l][: w.T].cpu().to(torch.float64).numpy()
        assert np.all(np.isfinite(got))
        for _ in range(60):
            i, h = int(rng.integers(w.B)), int(rng.integers(w.H))
            r = int(rng.integers(cu[i + 1] - cu[i]))
            _, o = oracle.attn_row(q, k, v, cu, i, h, r, w.scale, "f16")
            assert np.max(np.abs(got[cu[i] + r, h] - o)) <= 2e-3
    w = layers[-1]
    cu = hp.cu_from_lengths(w.lengths)
    want_x = oracle.unpack(wl.to_words(pipe.o[-1][: w.T].cpu()).reshape(w.T, w.C), w.keep.numpy(), cu, w.C, 1)
    assert np.array_equal(wl.to_words(pipe.x[-1].cpu()), want_x)


def test_one_launch_per_layer_loop_equals_the_three_launch_loop():
    """The 12 layers as 12 ragged_pack_attn_unpack launches in one graph: every cu_seqlens, every attention row and
    the final padded tensor equal the 36-kernel loop's bit for bit (which the tests above hold against the oracle)."""
    layers = _small_pipeline()
    ref = Pipeline(layers, fill_mode=1)
    ref.run()
    one = Pipeline(layers, fill_mode=1, one_launch=True)
    one.run()
    g = capture(torch, one.run)
    for rep in range(2):
        for t in one.x[1:] + one.o:
            t.fill_(9.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l, w in enumerate(layers):
            assert torch.equal(one.cu[l], ref.cu[l])
            assert torch.equal(one.gidx[l][: w.T], ref.gidx[l][: w.T])
            assert torch.equal(one.o[l][: w.T].view(torch.int16), ref.o[l][: w.T].view(torch.int16))
            assert torch.equal(one.x[l + 1].view(torch.int16), ref.x[l + 1].view(torch.int16))


def test_stay_packed_loop_matches_the_unpack_pack_loop_and_oracle():
    """Pack once, stay packed (strided attention, re-pack at the pruning layers, CLS read at the end):
    same lengths and attention rows as the loop that goes through the padded tensor every layer."""
    layers = _small_pipeline()
    ref = Pipeline(layers, fill_mode=1)
    ref.run()
    sp = StayPackedPipeline(layers)
    assert sp.prunes == [2, 5, 8] and sp.launches == 17
    sp.run()
    torch.cuda.synchronize()
    eager = ([o.clone() for o in sp.o], [c.clone() for c in sp.cu], sp.cls.clone(), [r.clone() for r in sp.rows])

    g = capture(torch, sp.run)
    for rep in range(3):
        for t in sp.o + sp.rows + [sp.cls]:
            t.fill_(5.0)
        for c in sp.cu:
            c.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for l in range(12):
            assert torch.equal(sp.o[l].view(torch.int16), eager[0][l].view(torch.int16))
        for a, b in zip(sp.cu, eager[1]):
            assert torch.equal(a, b)
        assert torch.equal(sp.cls.view(torch.int16), eager[2].view(torch.int16))

    # the same Q, K, V rows and lengths: attention outputs agree bit for bit with the padded-layout loop
    for l, w in enumerate(layers):
        assert torch.equal(sp.o[l][: w.T].view(torch.int16), ref.o[l][: w.T].view(torch.int16))
    stage_layers = [0, 2, 5, 8]
    for stage, l in enumerate(stage_layers):
        assert sp.cu[stage].cpu().numpy().tolist() == hp.cu_from_lengths(layers[l].lengths).tolist()
    # oracle: re-pack chain of layer outputs, composed gather index, CLS rows
    for stage, l in enumerate(stage_layers[1:], start=1):
        prev = layers[l - 1]
        rows = wl.to_words(sp.o[l - 1][: prev.T].cpu()).reshape(prev.T, prev.C)
        keep_rows = wl.pipeline_row_masks([w.keep for w in layers])[l].numpy()
        want_rows, want_cu, want_gi = oracle.repack(rows, keep_rows, hp.cu_from_lengths(prev.lengths))
        T = int(want_cu[-1])
        assert T == layers[l].T
        assert np.array_equal(sp.gidx[stage][:T].cpu().numpy(), want_gi)
    last = layers[-1]
    final_rows = wl.to_words(sp.o[-1][: last.T].cpu()).reshape(last.T, last.C)
    want_cls = oracle.cls_extract(final_rows, hp.cu_from_lengths(last.lengths))
    assert np.array_equal(wl.to_words(sp.cls.cpu()), want_cls)
    # CLS is never pruned, so the CLS row equals token 0 of the padded-layout loop's final tensor
    assert torch.equal(sp.cls.view(torch.int16), ref.x[-1][:, 0].contiguous().view(torch.int16))
    # the last re-pack's rows (written at layer 9 from layer 8's output)
    l = 8
    prev = layers[l - 1]
    rows = wl.to_words(sp.o[l - 1][: prev.T].cpu()).reshape(prev.T, prev.C)
    want_rows, _, _ = oracle.repack(rows, wl.pipeline_row_masks([w.keep for w in layers])[l].numpy(),
                                    hp.cu_from_lengths(prev.lengths))
    assert np.array_equal(wl.to_words(sp.rows[1][: layers[l].T].cpu()), want_rows)
