"""Measure every benchmark configuration on one MI355X and print one JSON line per case.

    python -m paper_2604_15408_amd.suite [--only CASE] [--out results/suite.jsonl]

Cases (each with the step issued as three launches and as the single ragged_pack_attn_unpack launch):
the headline batch (also with cold caches: many buffer sets in rotation); the bf16 pruning-ratio sweep next to a padded baseline of the same shape
(this library's own attention kernel run with every image at the full N tokens -- the bytes and
flops a padded dense attention has to spend, with no mask cost added); the 384x384 serving batches;
the 12-layer progressive-pruning loop captured in ONE HIP graph, both through the padded tensor every
layer (36 kernels) and staying packed (17 kernels); eight packed encoder blocks ("late blocks": LayerNorm,
QKV projection, ragged attention, output projection, MLP with GELU, residuals) with synthetic weights,
next to the same blocks over all B*N rows, and with three independent batches in flight on three streams.  Kernel times are HIP-event times
of a graph holding 20 back-to-back copies of the kernel (divided by 20), so they include the
in-graph kernel-to-kernel gap that an empty kernel shows separately.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

from . import workloads as wl
from .harness import (REPLICAS, PackedBlocks, PaddedPath, Path, Pipeline, ProgressiveBlocks, StayPackedPipeline, capture, pick_streams,
                      event_time_us, wall_steps)


def stage_times(torch, p: Path):
    out = {}
    for name, fn in (("pack", p.pack), ("attn", p.attn), ("unpack", p.unpack)):
        g = capture(torch, fn, REPLICAS)
        out[name] = event_time_us(torch, g.replay, iters=30)[0] / REPLICAS
    return out


def case(torch, w, label: str):
    p = Path(w, 0)
    alg = p.algorithmic()
    us = stage_times(torch, p)
    g = capture(torch, p.step)
    step_graph = wall_steps(torch, g.replay, 300) * 1e6
    lean = p.prepared_step()
    step_lean = wall_steps(torch, lean, 300) * 1e6
    g_one = capture(torch, p.one_launch, REPLICAS)
    one_us = event_time_us(torch, g_one.replay, iters=30)[0] / REPLICAS
    one_wall = wall_steps(torch, p.prepared_one_launch(), 300) * 1e6
    fused = PaddedPath(w, 0)
    g_fused = capture(torch, fused.run, REPLICAS)
    fused_us = event_time_us(torch, g_fused.replay, iters=30)[0] / REPLICAS
    fused_wall = wall_steps(torch, fused.prepared(), 300) * 1e6
    return {"case": label, "workload": w.name, "fused_single_launch_us": {"kernel": fused_us, "wall_prepared": fused_wall}, "dtype": w.dtype, "B": w.B, "N": w.N, "T": w.T,
            "max_len": max(w.lengths), "kernel_us": us,
            "gbs": {k: alg[k]["bytes"] / (us[k] * 1e-6) / 1e9 for k in us},
            "attn_tflops": alg["attn"]["flops"] / (us["attn"] * 1e-6) / 1e12,
            "attn_tokens_per_s": w.T / (us["attn"] * 1e-6),
            "step_us": {"hipgraph": step_graph, "eager_prepared": step_lean, "one_launch_prepared": one_wall},
            "one_launch_kernel_us": one_us,
            "step_tokens_per_s": w.T / (min(step_graph, step_lean, one_wall) * 1e-6)}


def cold_case(torch, w, label: str, sets: int):
    """The step and the attention kernel with caches that hold none of their data: `sets` copies of every
    buffer, used one after the other inside one graph, so that by the time a copy comes round again the
    other copies have pushed it out of the L2s and the 256 MB Infinity Cache.  (The other cases re-launch
    on the same buffers.)"""
    paths = [Path(w, 0) for _ in range(sets)]
    touched = paths[0].algorithmic()["pack_attn_unpack"]["bytes"]

    def all_steps():
        for p in paths:
            p.one_launch()

    def all_attn():
        for p in paths:
            p.attn()
    all_steps()
    torch.cuda.synchronize()
    us_step = event_time_us(torch, capture(torch, all_steps).replay, iters=20)[0] / sets
    us_attn = event_time_us(torch, capture(torch, all_attn).replay, iters=20)[0] / sets
    warm = paths[0]
    us_step_warm = event_time_us(torch, capture(torch, warm.one_launch, sets).replay, iters=20)[0] / sets
    us_attn_warm = event_time_us(torch, capture(torch, warm.attn, sets).replay, iters=20)[0] / sets
    return {"case": label, "workload": w.name, "T": w.T, "buffer_sets": sets,
            "touched_mb_all_sets": touched * sets / 1e6,
            "one_launch_us": {"cold": us_step, "warm": us_step_warm},
            "attn_us": {"cold": us_attn, "warm": us_attn_warm},
            "cold_step_tokens_per_s": w.T / (us_step * 1e-6)}


def padded_baseline(torch, w):
    """Attention time if every image kept all N tokens (what padding to N costs)."""
    full = wl.deit_b_pruned(1.0, w.B, w.dtype, w.seed)
    p = Path(full, 0)
    p.pack()
    torch.cuda.synchronize()
    g = capture(torch, p.attn, REPLICAS)
    return event_time_us(torch, g.replay, iters=30)[0] / REPLICAS


def library_padded_sdpa_us(torch, w):
    """Context only: the framework's own scaled_dot_product_attention on the padded [B, H, N, D] layout with
    a boolean key mask built from the keep mask -- what the paper calls the padded baseline.  Eager calls
    timed with events (the library call may allocate, so it is not captured).  None if the call fails."""
    try:
        import torch.nn.functional as F
        tdt = torch.float16 if w.dtype == "f16" else torch.bfloat16
        g = torch.Generator(device="cuda:0").manual_seed(1)
        q, k, v = (torch.randn(w.B, w.H, w.N, w.D, generator=g, device="cuda:0").to(tdt) for _ in range(3))
        mask = w.keep.to("cuda:0").bool()[:, None, None, :]              # keys of dropped tokens masked out
        fn = lambda: F.scaled_dot_product_attention(q, k, v, attn_mask=mask, scale=w.scale)
        return event_time_us(torch, lambda: [fn() for _ in range(10)], iters=20)[0] / 10
    except Exception:                                                    # noqa: BLE001 - optional context number
        return None


def pipeline_case(torch, one_launch: bool = False):
    layers = wl.pipeline()
    pipe = Pipeline(layers, fill_mode=1, one_launch=one_launch)
    pipe.run()
    torch.cuda.synchronize()
    g = capture(torch, pipe.run)
    us_graph = event_time_us(torch, g.replay, iters=30)[0]
    wall_graph = wall_steps(torch, g.replay, 100) * 1e6
    wall_eager = wall_steps(torch, pipe.run, 100) * 1e6
    return {"case": "pipeline_12_layers" + ("_one_launch_per_layer" if one_launch else ""), "B": layers[0].B, "N": layers[0].N,
            "T_per_layer": [w.T for w in layers], "tokens": pipe.tokens, "kernels_in_graph": pipe.launches,
            "graph_gpu_us": us_graph, "graph_wall_us": wall_graph, "eager_wall_us": wall_eager,
            "tokens_per_s": pipe.tokens / (wall_graph * 1e-6)}


def stay_packed_case(torch):
    layers = wl.pipeline()
    pipe = StayPackedPipeline(layers)
    pipe.run()
    torch.cuda.synchronize()
    g = capture(torch, pipe.run)
    us_graph = event_time_us(torch, g.replay, iters=30)[0]
    wall_graph = wall_steps(torch, g.replay, 100) * 1e6
    wall_eager = wall_steps(torch, pipe.run, 100) * 1e6
    return {"case": "pipeline_12_layers_stay_packed", "B": layers[0].B, "N": layers[0].N,
            "T_per_layer": [w.T for w in layers], "tokens": pipe.tokens, "kernels_in_graph": pipe.launches,
            "graph_gpu_us": us_graph, "graph_wall_us": wall_graph, "eager_wall_us": wall_eager,
            "tokens_per_s": pipe.tokens / (wall_graph * 1e-6)}


def late_blocks_case(torch, w, label: str, depth: int = 8, tight_cap: bool = False, keep_prob: float | None = None):
    """pack + `depth` encoder blocks on the packed rows + CLS read, in one HIP graph, next to the same
    blocks over all B*N rows (what a padded pipeline computes).  keep_prob: the pruning ratio the caller
    configured; the expected row count B * (1 + (N-1) * keep_prob) goes to the linear layers as a hint."""
    hint = 0 if keep_prob is None else int(round(w.B * (1 + (w.N - 1) * keep_prob)))

    def timed(workload):
        pb = PackedBlocks(workload, depth, rows_cap=workload.T if tight_cap else None,
                          rows_hint=hint if workload is w else 0)
        pb.run()
        torch.cuda.synchronize()
        g = capture(torch, pb.run)
        gpu_us = event_time_us(torch, g.replay, iters=20)[0]
        return pb, gpu_us, wall_steps(torch, g.replay, 50) * 1e6
    pb, gpu_us, wall_us = timed(w)
    full = wl.deit_b_pruned(1.0, w.B, w.dtype, w.seed) if w.N == 197 else None
    rec = {"case": label, "workload": w.name, "B": w.B, "N": w.N, "T": w.T, "depth": depth,
           "rows_cap": w.T if tight_cap else w.B * w.N, "rows_hint": hint,
           "kernels_in_graph": pb.launches, "graph_gpu_us": gpu_us, "graph_wall_us": wall_us,
           "us_per_block": gpu_us / depth, "tflops": pb.flops() / gpu_us / 1e6,
           "tokens_per_s": w.T * depth / (wall_us * 1e-6), "images_per_s_through_late_blocks": w.B / (wall_us * 1e-6)}
    if full is not None and full.T != w.T:
        _, pad_us, _ = timed(full)
        rec["padded_graph_gpu_us"] = pad_us
        rec["speedup_vs_padded"] = pad_us / gpu_us
    return rec


def in_flight(torch, make, batches: int, steps: int = 40):
    """Wall time per batch with `batches` independent pipelines in flight: one graph per pipeline (make()
    returns an object with run()), each replayed on its own HIP stream (default priority, chosen by
    pick_streams), against one pipeline alone."""
    graphs = []
    for _ in range(batches):
        obj = make()
        obj.run()
        torch.cuda.synchronize()
        graphs.append((capture(torch, obj.run), obj))

    def bind(selection):
        def go():
            for (g, _), st in zip(graphs, selection):
                with torch.cuda.stream(st):
                    g.replay()
        return go
    _, go = pick_streams(torch, batches, bind, burst=10)
    for _ in range(5):
        go()
    return wall_steps(torch, go, steps) / batches, wall_steps(torch, graphs[0][0].replay, steps)


def late_blocks_in_flight_case(torch, w, label: str, batches: int, keep_prob: float, depth: int = 8):
    """Several independent batches in flight through the packed blocks.  At a few thousand rows every kernel
    of the block is bound by latency and leaves most of the chip idle, so kernels of different batches overlap."""
    hint = int(round(w.B * (1 + (w.N - 1) * keep_prob)))
    per_batch, one = in_flight(torch, lambda: PackedBlocks(w, depth, rows_hint=hint), batches)
    return {"case": label, "workload": w.name, "B": w.B, "T": w.T, "depth": depth, "batches_in_flight": batches,
            "wall_us_per_batch": per_batch * 1e6, "wall_us_per_batch_alone": one * 1e6,
            "images_per_s_through_late_blocks": w.B / per_batch, "tokens_per_s": w.T * depth / per_batch}


def progressive_case(torch, B: int, label: str):
    """A 12-block DeiT-B-shaped encoder that prunes to 70 % by top-k l2 score in front of blocks 3, 6 and 9
    (197 -> 138 -> 97 -> 68 tokens per image) and stays packed throughout, in one HIP graph; next to the same
    12 blocks without pruning."""
    def timed(prune_at):
        pb = ProgressiveBlocks(B=B, depth=12, prune_at=prune_at, keep_ratio=0.7)
        pb.run()
        torch.cuda.synchronize()
        g = capture(torch, pb.run)
        return pb, event_time_us(torch, g.replay, iters=10)[0], wall_steps(torch, g.replay, 20) * 1e6
    pb, gpu_us, wall_us = timed((3, 6, 9))
    _, dense_us, _ = timed(())
    per_batch, _ = in_flight(torch, lambda: ProgressiveBlocks(B=B, depth=12, prune_at=(3, 6, 9), keep_ratio=0.7), 3, steps=15)
    return {"case": label, "B": B, "N": pb.N, "tokens_per_image": pb.lengths, "kernels_in_graph": pb.launches,
            "graph_gpu_us": gpu_us, "graph_wall_us": wall_us, "unpruned_graph_gpu_us": dense_us,
            "speedup_vs_unpruned": dense_us / gpu_us, "token_blocks": pb.tokens(),
            "images_per_s": B / (wall_us * 1e-6), "wall_us_per_batch_3_in_flight": per_batch * 1e6,
            "images_per_s_3_in_flight": B / per_batch}


def prune_once_case(torch, B: int, H: int, label: str):
    """The paper's Section 4.3 schedule on a 12-block encoder of DeiT width H*64 with synthetic weights: four
    blocks on all tokens, one pruning stage (top-k l2 score) in front of block 4, eight blocks on the packed
    rows, class tokens read from the packed buffer -- for several keep ratios, one HIP graph each."""
    out = {"case": label, "B": B, "C": H * 64, "N": 197, "graph_gpu_us": {}, "images_per_s": {}, "tokens_after_pruning": {}}
    for ratio in (1.0, 0.5, 0.2, 0.1):
        pb = ProgressiveBlocks(B=B, H=H, depth=12, prune_at=() if ratio == 1.0 else (4,), keep_ratio=ratio)
        pb.run()
        torch.cuda.synchronize()
        g = capture(torch, pb.run)
        us = event_time_us(torch, g.replay, iters=10)[0]
        key = f"keep_{ratio}"
        out["graph_gpu_us"][key] = us
        out["images_per_s"][key] = B / (us * 1e-6)
        out["tokens_after_pruning"][key] = pb.lengths[-1]
    base = out["graph_gpu_us"]["keep_1.0"]
    out["speedup_vs_unpruned"] = {k: base / v for k, v in out["graph_gpu_us"].items()}
    return out


LINEAR_LAYERS = (("qkv", 2304, 768, "none"), ("out", 768, 768, "none"), ("fc1", 3072, 768, "gelu"), ("fc2", 768, 3072, "none"))


def linear_case(torch, rows: int, shape=None, library: bool = True):
    """ragged_linear alone on the four layer shapes of a DeiT-B block at `rows` rows (bias; GELU on fc1): us per
    launch in a graph of 10 and TFLOP/s; for context the framework library's GEMM (torch.addmm, no GELU) on
    the same shape.  shape = (N, K) restricts the run to one layer shape (used under the profiler)."""
    from . import binding
    dev = "cuda:0"
    rec = {"case": "linear_layers", "rows": rows, "us": {}, "tflops": {}, "library_addmm_us": {}}
    layers = [("custom", shape[0], shape[1], "none")] if shape else LINEAR_LAYERS
    for name, N, K, act in layers:
        g = torch.Generator(device=dev).manual_seed(rows + N)
        x = torch.randn(rows, K, generator=g, device=dev).half()
        w = (torch.randn(N, K, generator=g, device=dev) * K ** -0.5).half()
        b = torch.randn(N, generator=g, device=dev).half()
        y = torch.zeros(rows, N, device=dev).half()
        fn = lambda: binding.ragged_linear(x, w, b, None, y, None, act)
        us = event_time_us(torch, capture(torch, fn, 10).replay, iters=20)[0] / 10
        rec["us"][name], rec["tflops"][name] = us, 2 * rows * N * K / us / 1e6
        if library:
            wt = w.t().contiguous()
            lib = lambda: torch.addmm(b, x, wt, out=y)
            for _ in range(3):
                lib()
            torch.cuda.synchronize()
            rec["library_addmm_us"][name] = event_time_us(torch, capture(torch, lib, 10).replay, iters=20)[0] / 10
    return rec


def mask_producer_case(torch, B: int = 32, N: int = 197, k: int = 40):
    """The keep-mask producer in front of pack: fp64 l2 scores + per-image top-k, then pack."""
    from . import binding
    dev = "cuda:0"
    x = wl.deit_b_pruned(1.0, B, "f16", 1008).features().to(dev)
    C = x.shape[2]
    scores = torch.zeros(B, N, dtype=torch.float64, device=dev)
    keep = torch.zeros(B, N, dtype=torch.uint8, device=dev)
    out = {}
    for name, fn in (("token_scores_l2", lambda: binding.ragged_token_scores_l2(x, scores)),
                     ("keep_topk", lambda: binding.ragged_keep_topk(scores, k, keep))):
        g = capture(torch, fn, REPLICAS)
        out[name] = event_time_us(torch, g.replay, iters=30)[0] / REPLICAS
    return {"case": "mask_producer", "B": B, "N": N, "C": C, "k": k, "kernel_us": out,
            "scores_gbs": B * N * C * 2 / (out["token_scores_l2"] * 1e-6) / 1e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=None)
    ap.add_argument("--only", default=None, help="run only the cases whose name starts with this (e.g. late_blocks)")
    ap.add_argument("--linear-shape", default=None, metavar="ROWS,N,K",
                    help="with --only linear: one ragged_linear shape only, without the library GEMM (for the profiler)")
    args = ap.parse_args()
    import torch
    from . import binding
    if not torch.cuda.is_available():
        raise SystemExit("the suite needs a GPU")
    binding.load()
    lines = []

    def emit(rec):
        lines.append(rec)
        print(json.dumps(rec), flush=True)

    def want(name):
        return args.only is None or name.startswith(args.only)

    if want("headline"):
        emit(case(torch, wl.deit_b_pruned(0.2, 32, "f16", 1001), "headline"))
    if want("cold"):
        emit(cold_case(torch, wl.deit_b_pruned(0.2, 32, "f16", 1001), "cold_headline", sets=32))
        emit(cold_case(torch, wl.pipeline()[0], "cold_dense_bs64", sets=6))
    if want("uniform"):
        # the paper's kernel-latency table (Section 3): BS 32 and 64 at 0 / 50 / 80 % pruning = 197 / 99 / 40 tokens per image
        for B in (32, 64):
            for per_image in (197, 99, 40):
                emit(case(torch, wl.uniform(B, per_image), "uniform_lengths"))
        emit(case(torch, wl.uniform(1, 40), "uniform_lengths"))
    if want("mask_producer"):
        emit(mask_producer_case(torch))
    if want("sweep"):
        pad_us = None
        for w in wl.sweep():
            rec = case(torch, w, "sweep")
            if pad_us is None:
                pad_us = padded_baseline(torch, w)
            rec["padded_attn_us"] = pad_us
            rec["library_padded_sdpa_us"] = library_padded_sdpa_us(torch, w)
            rec["attn_speedup_vs_padded"] = pad_us / rec["kernel_us"]["attn"]
            emit(rec)
    if want("serving_384"):
        for B in (1, 2, 4, 32):
            emit(case(torch, wl.serving_384(B), "serving_384"))
    if want("pipeline"):
        emit(pipeline_case(torch))
        emit(pipeline_case(torch, one_launch=True))
        emit(stay_packed_case(torch))
    if want("late_blocks"):
        emit(late_blocks_case(torch, wl.deit_b_pruned(0.2, 32, "f16", 1001), "late_blocks_headline", keep_prob=0.2))
        emit(late_blocks_in_flight_case(torch, wl.deit_b_pruned(0.2, 32, "f16", 1001), "late_blocks_headline_3_in_flight",
                                        batches=3, keep_prob=0.2))
        # a fixed number of kept tokens per image: T is known on the host and is the row capacity
        emit(late_blocks_case(torch, wl.uniform(32, 40), "late_blocks_uniform40_tight_cap", tight_cap=True))
        emit(late_blocks_case(torch, wl.deit_b_pruned(0.5, 8, "f16", 1005), "late_blocks_bs8_keep0.5", keep_prob=0.5))
        emit(late_blocks_case(torch, wl.deit_b_pruned(1.0, 64, "f16", 1006), "late_blocks_bs64_dense"))
    if want("linear"):
        if args.linear_shape:
            rows, N, K = (int(v) for v in args.linear_shape.split(","))
            emit(linear_case(torch, rows, (N, K), library=False))
        else:
            for rows in (12608, 6304, 1334):
                emit(linear_case(torch, rows))
    if want("prune_once"):
        for H, name in ((12, "base"), (6, "small"), (3, "tiny")):
            emit(prune_once_case(torch, 32, H, f"prune_once_deit_{name}_bs32"))
        emit(prune_once_case(torch, 8, 12, "prune_once_deit_base_bs8"))
        emit(prune_once_case(torch, 128, 12, "prune_once_deit_base_bs128"))
    if want("progressive"):
        emit(progressive_case(torch, 32, "progressive_12_blocks_bs32"))
        emit(progressive_case(torch, 8, "progressive_12_blocks_bs8"))
    if args.out:
        os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
        with open(args.out, "w") as f:
            for rec in lines:
                f.write(json.dumps(rec) + "\n")


if __name__ == "__main__":
    sys.exit(main())
