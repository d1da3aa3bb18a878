"""Benchmark of the pack -> ragged attention -> unpack hot path on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--report PATH]

A "step" is one pass of the whole path over one synthetic batch: ragged_pack (keep mask ->
cu_seqlens, gather indices, packed rows), ragged_attn on seeded Q/K/V of the packed length using
the cu_seqlens pack just wrote, ragged_unpack of the attention output with pack's gather indices --
issued either as those three launches or as ragged_pack_attn_unpack, one launch that produces the
same outputs bit for bit.  The reported `value` is the single-launch entry point called back to back on
ONE stream with pre-marshalled arguments; the other ways of issuing the step are in extras.
Timing: after W untimed steps, 31 blocks of back-to-back steps (a multiple of K, at least 1000), each
between two device synchronisations; median, p10 and p90 over the blocks.
Inputs are resident in HBM before the timed region.  The default workload is the headline one:
DeiT-Base attention geometry (N=197, H=12, D=64), B=32, 80 % pruned (keep probability 0.2), fp16.

The single JSON line printed at the end carries, beside the whole-path throughput, the roofline of
the dominant kernel (timed live with HIP events over graph replays of that kernel alone; warm and with
cold caches; against the published peak and against a streaming copy measured in the same run), the
per-stage kernel times, the launch floor, a compact record of every other benchmark configuration, and
the CPU oracle timed on this machine's host cores (one thread and all of them).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2604_15408_amd.harness import (BLOCKS, HBM_PEAK_GBS, MFMA_F16_PEAK_TFLOPS, REPLICAS, Ceilings, ColdSets,  # noqa: E402
                                          PaddedPath, Path, Pipeline, StayPackedPipeline, StreamedSteps, algorithmic,
                                          block_steps, capture, config_point, kernel_time_us, make_workload,
                                          pipeline_point, spread, timed_blocks, wall_blocks, wall_steps)

HEADLINE_MODE = "one_launch_prepared"     # the step whose time is reported: one launch, one stream


def cpu_baseline(w, fill_mode: int):
    """The CPU oracle on the same workload: one thread, and all host cores available to this process.
    Only calls into the oracle are inside the timed regions (the fp64 -> 16-bit conversion of the attention
    output that unpack consumes is done between them, untimed)."""
    import torch
    import oracle
    from paper_2604_15408_amd import workloads as wl
    tdt = torch.float16 if w.dtype == "f16" else torch.bfloat16
    cores = min(len(os.sched_getaffinity(0)), oracle.max_threads())
    x = wl.to_words(w.features())
    keep = w.keep.numpy()
    q, k, v = (wl.to_words(t) for t in w.qkv())

    def once(threads: int) -> float:
        t0 = time.perf_counter()
        packed, cu, gidx = oracle.pack(x, keep)
        o = oracle.attn(q, k, v, cu, w.scale, w.dtype, threads=threads)
        t1 = time.perf_counter()
        o16 = wl.to_words(torch.from_numpy(o).to(tdt)).reshape(-1, w.C)
        t2 = time.perf_counter()
        oracle.unpack(o16, keep, cu, w.C, fill_mode)
        return (t1 - t0) + (time.perf_counter() - t2)
    t_all = statistics.median(once(cores) for _ in range(5))
    t_one = statistics.median(once(1) for _ in range(3))
    return {"value": w.T / t_all, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "ms_per_step": t_all * 1e3,
            "single_thread": {"value": w.T / t_one, "unit": "tokens/s", "cores": 1, "ms_per_step": t_one * 1e3},
            "sample": f"whole {w.name} batch (T={w.T}), pack+attn+unpack, median of 5 runs (all cores) "
                      "and of 3 runs (one thread)"}


def other_configs(torch, steps: int):
    """Every other benchmark configuration, compactly: the tiny case, the bf16 pruning-ratio sweep with its padded
    baseline (the same kernel with every image at all N tokens), the 384x384 serving batches, and the 12-layer
    progressive-pruning loop as one HIP graph (through the padded tensor every layer, and staying packed)."""
    from paper_2604_15408_amd import workloads as wl
    out = {"tiny": config_point(torch, wl.tiny(), steps)}
    sweep = [config_point(torch, w, steps) for w in wl.sweep()]
    padded_us = sweep[0]["attn_us"]                    # keep 1.0: every image at N tokens = the padded shape
    for rec in sweep:
        rec["attn_speedup_vs_padded"] = padded_us / rec["attn_us"]
    out["sweep_bf16"] = {"keep_probs": list(wl.SWEEP_KEEP_PROBS), "padded_attn_us": padded_us, "points": sweep}
    out["serving_384"] = [config_point(torch, wl.serving_384(B), steps) for B in (1, 2, 4, 32)]
    layers = wl.pipeline()
    alg = sum(algorithmic(w, 1)[k]["bytes"] for w in layers for k in ("pack", "attn", "unpack"))
    out["pipeline_12_layers"] = {
        "B": layers[0].B, "T_per_layer": [w.T for w in layers],
        "pack_attn_unpack_per_layer": pipeline_point(torch, Pipeline(layers, fill_mode=1), 36, alg),
    }
    fused_alg = sum(algorithmic(w, 1)["pack_attn_unpack"]["bytes"] for w in layers)
    out["pipeline_12_layers"]["one_launch_per_layer"] = pipeline_point(torch, Pipeline(layers, fill_mode=1, one_launch=True),
                                                                       12, fused_alg)
    stay = StayPackedPipeline(layers)
    out["pipeline_12_layers"]["stay_packed"] = pipeline_point(torch, stay, stay.launches)
    return out


def run(args):
    import torch
    from paper_2604_15408_amd import binding
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (there is no CPU fallback of the product path)")
    binding.load()
    w = make_workload(args.workload)
    p = Path(w, args.fill_mode)
    alg = p.algorithmic()

    # ---- whole path (every output of pack, attn and unpack).  The reported step is HEADLINE_MODE: the
    # single-launch entry point with pre-marshalled arguments, back to back on ONE stream.  Beside it:
    #   hipgraph            one hipGraphLaunch of the captured three-kernel pipeline
    #   eager               three checked binding calls (tensor checks + marshalling every call)
    #   eager_prepared      three calls with pre-marshalled arguments
    #   one_launch          ragged_pack_attn_unpack, checked call
    #   streams3            independent batches (own buffers) round-robin on three streams: a throughput of
    #                       overlapping batches, not a step time
    # Every way: W untimed steps, then BLOCKS blocks of block_steps(K) steps, median / p10 / p90 over the blocks.
    g_step = capture(torch, p.step)
    streamed = StreamedSteps(w, args.fill_mode, streams=3, tune=False)
    issue = {"one_launch_prepared": p.prepared_one_launch(), "one_launch": p.one_launch,
             "eager_prepared": p.prepared_step(), "eager": p.step, "hipgraph": g_step.replay,
             "streams3_one_launch_prepared": streamed.step}
    t_modes, gpu_modes, enq_modes = {}, {}, {}
    for name, fn in issue.items():
        for _ in range(args.warmup):
            fn()
        if name.startswith("streams3"):               # events on one stream see only a third of these launches
            t_modes[name] = wall_blocks(torch, fn, args.steps, args.blocks)
        else:
            t_modes[name], gpu_modes[name], enq_modes[name] = timed_blocks(torch, fn, args.steps, args.blocks,
                                                                           with_enqueue=True)
    t_step = t_modes[HEADLINE_MODE]["median"]

    # ---- each kernel alone: REPLICAS back-to-back copies in one graph, HIP events around each replay
    stage = {name: kernel_time_us(torch, fn) for name, fn in
             (("pack", p.pack), ("attn", p.attn), ("unpack", p.unpack), ("pack_attn_unpack", p.one_launch))}
    stage_us = {k: v["median"] for k, v in stage.items()}
    pipe_us = kernel_time_us(torch, p.step)["median"]

    # ---- the same kernel with caches that hold none of its data (32 buffer sets in rotation, ~460 MB per round)
    cold = ColdSets(w, 32, args.fill_mode)
    cold_step = cold.time_us(torch, "one_launch")
    cold_attn = cold.time_us(torch, "attn")
    del cold

    # ---- the same layer as ONE launch on the padded layout (gather-on-load attention)
    fused = PaddedPath(w, args.fill_mode)
    fused_kernel_us = kernel_time_us(torch, fused.run)["median"]
    fused_wall = wall_blocks(torch, fused.prepared(), args.steps, 7)

    # ---- launch floor: an empty kernel, same grid size as the attention launch
    attn_grid = w.B * w.H * ((w.N + 63) // 64)
    noop = lambda: binding.ragged_noop(attn_grid)
    g_noop1 = capture(torch, noop, 1)
    floor = {
        "noop_kernel_in_graph_us": kernel_time_us(torch, noop, iters=20)["median"],
        "noop_eager_wall_us": wall_steps(torch, lambda: (noop(), torch.cuda.synchronize()), 200) * 1e6,
        "noop_graph_launch_wall_us": wall_steps(torch, lambda: (g_noop1.replay(), torch.cuda.synchronize()), 200) * 1e6,
        "noop_eager_enqueue_us": wall_steps(torch, noop, 1000) * 1e6,
        "attn_eager_wall_us": wall_steps(torch, lambda: (p.attn(), torch.cuda.synchronize()), 200) * 1e6,
        "attn_eager_enqueue_us": wall_steps(torch, p.attn, 1000) * 1e6,
    }

    ceilings = Ceilings().measure(torch)

    # HBM traffic per launch comes from rocprofv3 --pmc passes made offline over this same command
    # (a counter run cannot share a process with timing); null if this workload was not profiled.
    traffic = {}
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            traffic = json.load(f).get(w.name, {})
    except OSError:
        pass
    # the kernel the reported step runs in; its average launch duration is the HIP-event time of the timed
    # blocks of the reported step themselves (mean over the blocks), one launch per step
    dominant = "pack_attn_unpack"
    dom = gpu_modes[HEADLINE_MODE]
    dom_us = dom["mean"]
    achieved = alg[dominant]["bytes"] / (dom_us * 1e-6) / 1e9
    achieved_cold = alg[dominant]["bytes"] / (cold_step["mean"] * 1e-6) / 1e9
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": traffic.get(dominant, {}).get("hbm_bytes"),
                "avg_launch_us": dom_us, "launch_us_p10_p90": [dom["p10"], dom["p90"]],
                "in_graph_launch_us": stage[dominant]["mean"],
                "algorithmic_bytes": alg[dominant]["bytes"],
                "cold_launch_us": cold_step["mean"], "achieved_cold": achieved_cold,
                "frac_cold": achieved_cold / HBM_PEAK_GBS,
                "achievable": ceilings["hbm_copy_gbs"], "frac_of_achievable": achieved / ceilings["hbm_copy_gbs"],
                "cache_state": "frac: the same buffers re-launched (reads served by the 256 MB Infinity Cache); "
                               "frac_cold: 32 buffer sets in rotation"}
    attn_tflops = alg["attn"]["flops"] / (stage_us["attn"] * 1e-6) / 1e12

    result = {
        "metric": "packed tokens/s through pack+ragged_attn+unpack (DeiT-B shape, 80% pruned, BS=32); ragged_attn us/call in extras",
        "value": w.T / t_step, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": t_step * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "N": w.N, "H": w.H, "D": w.D, "T": w.T,
                   "max_len": max(w.lengths), "lengths": w.note, "launch": HEADLINE_MODE,
                   "streams": 1, "unpack_fill_mode": args.fill_mode},
        "timing": {"blocks": args.blocks, "steps_per_block": block_steps(args.steps),
                   "ms_per_step_p10": t_modes[HEADLINE_MODE]["p10"] * 1e3,
                   "ms_per_step_p90": t_modes[HEADLINE_MODE]["p90"] * 1e3,
                   "host_enqueue_us_per_step": enq_modes[HEADLINE_MODE]["median"] * 1e6,
                   "note": "value and ms_per_step are the median over the blocks; each block is a multiple of "
                           "--steps back-to-back steps between two device synchronisations; host_enqueue_us_per_step "
                           "is the host time per call until the block's last call has returned (when it is as long "
                           "as the step, the Python call rate bounds the block, not the kernel: the same loop from "
                           "C++, ragged_call_cost, is the check)"},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline(w, args.fill_mode),
        "extras": {
            "ragged_attn_us_per_call": stage_us["attn"],
            "ragged_attn_tokens_per_s": w.T / (stage_us["attn"] * 1e-6),
            "kernel_us": stage_us,
            "kernel_us_p10_p90": {k: [v["p10"], v["p90"]] for k, v in stage.items()},
            "pipeline_kernels_us": pipe_us,
            "step_wall_us": {k: v["median"] * 1e6 for k, v in t_modes.items()},
            "step_wall_us_p10_p90": {k: [v["p10"] * 1e6, v["p90"] * 1e6] for k, v in t_modes.items()},
            "step_gpu_us": {k: v["median"] for k, v in gpu_modes.items()},
            "attn_mfma_tflops": attn_tflops, "attn_mfma_frac": attn_tflops / MFMA_F16_PEAK_TFLOPS,
            "stage_gbs": {k: alg[k]["bytes"] / (stage_us[k] * 1e-6) / 1e9 for k in stage_us},
            "cold_kernel_us": {"pack_attn_unpack": cold_step["median"], "attn": cold_attn["median"]},
            "three_launch_tokens_per_s": w.T / min(t_modes[k]["median"] for k in ("hipgraph", "eager", "eager_prepared")),
            "streams3_throughput": {"tokens_per_s": w.T / t_modes["streams3_one_launch_prepared"]["median"],
                                    "streams": 3, "note": "independent batches overlapping on three streams; "
                                                          "a throughput, not a step time"},
            "fused_single_launch": {"entry": "ragged_attn_padded", "kernel_us": fused_kernel_us,
                                    "wall_us_per_layer": fused_wall["median"] * 1e6,
                                    "tokens_per_s": w.T / fused_wall["median"]},
            "floor": floor,
            "ceilings": ceilings,
            "paper_context": "paper's Triton kernel on RTX 4000 Ada: 24 us attention latency at BS=32, 40 tok/img (uniform lengths)",
        },
    }
    if not args.no_configs:
        result["extras"]["configs"] = other_configs(torch, args.steps)
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="headline")
    ap.add_argument("--fill-mode", type=int, default=0, choices=(0, 1))
    ap.add_argument("--report", default=None, help="also write the JSON to this path")
    ap.add_argument("--blocks", type=int, default=BLOCKS,
                    help="timed blocks per way of issuing the step (median / p10 / p90 are taken over them)")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the compact block on the other benchmark configurations (used under the profiler)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 64 MiB elementwise copy kernel (known traffic) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (images are independent, so the path "
              "shards by image with no exchange step); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    result = run(args)
    if args.calibrate_copy:
        import torch
        src = torch.arange(16 << 20, dtype=torch.int32, device="cuda:0")      # 64 MiB
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1, out=dst)                                        # reads 64 MiB, writes 64 MiB
        torch.cuda.synchronize()
    line = json.dumps(result)
    if args.report:
        os.makedirs(os.path.dirname(os.path.abspath(args.report)), exist_ok=True)
        with open(args.report, "w") as f:
            f.write(line + "\n")
    print(line)


if __name__ == "__main__":
    main()
