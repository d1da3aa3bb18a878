"""Measurement plumbing shared by ``bench.py`` and ``paper_2604_15408_amd.suite``: device buffers for a
workload, the three stage calls, HIP-graph capture and event timing.  No arithmetic of the method.
"""
from __future__ import annotations

import statistics
import time

REPLICAS = 20                    # copies of one kernel inside a graph when timing that kernel alone
BLOCKS = 31                      # timed blocks per measurement: median, p10 and p90 are taken over these
MIN_BLOCK_STEPS = 1000           # a block lasts at least this many steps (several ms at ViT sizes)
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0    # dense fp16/bf16 MFMA, published


def spread(samples):
    """median, 10th / 90th percentile and mean of a list of samples."""
    xs = sorted(samples)
    n = len(xs)
    pick = lambda f: xs[min(n - 1, max(0, int(round(f * (n - 1)))))]
    return {"median": statistics.median(xs), "p10": pick(0.10), "p90": pick(0.90), "mean": statistics.fmean(xs)}


def block_steps(steps: int) -> int:
    """Steps per timed block: the smallest multiple of `steps` that reaches MIN_BLOCK_STEPS."""
    steps = max(1, int(steps))
    return steps * -(-MIN_BLOCK_STEPS // steps)


def wall_blocks(torch, fn, steps: int, blocks: int = BLOCKS):
    """Wall-clock seconds per step of fn(): `blocks` blocks of block_steps(steps) back-to-back calls, each
    block bracketed by a device synchronisation; returns spread() over the per-block averages."""
    n = block_steps(steps)
    return spread([wall_steps(torch, fn, n) for _ in range(blocks)])


def timed_blocks(torch, fn, steps: int, blocks: int = BLOCKS, with_enqueue: bool = False):
    """wall_blocks() with a pair of HIP events recorded on the launching stream around the calls of every
    block as well: returns (wall seconds per step, GPU microseconds per step between the two events), both as
    spread() over the blocks; with_enqueue adds the host seconds per step until the last call of a block has
    returned (before the synchronisation): where that equals the wall time, the host's call rate and not the
    kernel is what the block measured.  The event time is the average duration of one launch inside the timed region,
    including whatever gap the stream leaves between consecutive kernels."""
    n = block_steps(steps)
    wall, gpu, enq = [], [], []
    for _ in range(blocks):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        t_enq = time.perf_counter()
        torch.cuda.synchronize()
        wall.append((time.perf_counter() - t0) / n)
        enq.append((t_enq - t0) / n)
        gpu.append(e0.elapsed_time(e1) * 1e3 / n)
    if with_enqueue:
        return spread(wall), spread(gpu), spread(enq)
    return spread(wall), spread(gpu)


def make_workload(name: str):
    from paper_2604_15408_amd import workloads as wl
    if name == "headline":
        return wl.deit_b_pruned(0.2, 32, "f16", 1001)
    if name == "tiny":
        return wl.tiny()
    if name.startswith("keep"):                       # e.g. keep0.6 : bf16 sweep point
        p = float(name[4:])
        k = wl.SWEEP_KEEP_PROBS.index(p)
        return wl.sweep()[k]
    if name.startswith("serving"):                    # e.g. serving4
        return wl.serving_384(int(name[7:]))
    if name.startswith("layer"):                      # e.g. layer1 : pipeline layer (B=64)
        return wl.pipeline()[int(name[5:]) - 1]
    raise SystemExit(f"unknown workload {name!r}")


class Path:
    """Device buffers of one workload plus the three stage calls."""

    def __init__(self, w, fill_mode: int = 0):
        import torch
        from paper_2604_15408_amd import binding
        self.torch, self.b, self.w, self.fill_mode = torch, binding, w, fill_mode
        dev = "cuda:0"
        B, N, C, H, D = w.B, w.N, w.C, w.H, w.D
        self.T = w.T
        cap = B * N                                    # row capacity of every packed buffer
        self.x = w.features().to(dev)
        self.keep = w.keep.to(dev)
        self.packed = torch.zeros(cap, C, dtype=self.x.dtype, device=dev)
        self.cu = torch.zeros(B + 1, dtype=torch.int32, device=dev)
        self.gidx = torch.zeros(cap, dtype=torch.int32, device=dev)
        self.q, self.k, self.v = (torch.zeros(cap, H, D, dtype=self.x.dtype, device=dev) for _ in range(3))
        for dst, src in zip((self.q, self.k, self.v), w.qkv(max(self.T, 1))):
            dst[: src.shape[0]] = src.to(dev)          # rows past T are never read
        self.o = torch.zeros(cap, H, D, dtype=self.q.dtype, device=dev)
        self.out = torch.zeros(B, N, C, dtype=self.x.dtype, device=dev)
        torch.cuda.synchronize()

    def pack(self):
        self.b.ragged_pack(self.x, self.keep, self.packed, self.cu, self.gidx)

    def attn(self):
        # max_seqlen = N: nothing about the lengths is known on the host (no sync after pack)
        self.b.ragged_attn(self.q, self.k, self.v, self.o, self.cu, self.w.N, self.w.scale)

    def unpack(self):
        self.b.ragged_unpack(self.o.view(-1, self.w.C), self.keep, self.cu, self.gidx, self.out,
                             self.fill_mode)

    def step(self):
        self.pack()
        self.attn()
        self.unpack()

    def one_launch(self):
        """The same step -- every output of pack, attn and unpack -- as a single launch."""
        self.b.ragged_pack_attn_unpack(self.x, self.keep, self.q, self.k, self.v, self.packed, self.cu,
                                       self.gidx, self.o, self.out, self.w.scale, self.fill_mode)

    def prepared_one_launch(self):
        return self.b.prepare_pack_attn_unpack(self.x, self.keep, self.q, self.k, self.v, self.packed, self.cu,
                                               self.gidx, self.o, self.out, self.w.scale, self.fill_mode)

    def prepared_step(self):
        """The same three launches with arguments marshalled once (binding.Prepared), bound to the
        current stream: what a serving loop that re-launches fixed buffers would call."""
        b, w = self.b, self.w
        calls = (b.prepare_pack(self.x, self.keep, self.packed, self.cu, self.gidx),
                 b.prepare_attn(self.q, self.k, self.v, self.o, self.cu, w.N, w.scale),
                 b.prepare_unpack(self.o.view(-1, w.C), self.keep, self.cu, self.gidx, self.out,
                                  self.fill_mode))

        def step():
            for call in calls:
                call()
        return step

    def algorithmic(self):
        return algorithmic(self.w, self.fill_mode)


def algorithmic(w, fill_mode: int = 0):
    """Algorithmic bytes / flops of one launch of each stage (what the method itself must move)."""
    T = w.T
    row = w.C * 2
    sq = sum(n * n for n in w.lengths)
    unpack_bytes = 2 * T * row + 4 * T if fill_mode == 0 else T * row + w.B * w.N * row + w.B * w.N
    stages = {
        "pack": {"bytes": w.B * w.N + 2 * T * row + 4 * (w.B + 1) + 4 * T},
        "attn": {"bytes": 4 * T * row, "flops": 4 * w.D * w.H * sq},
        "unpack": {"bytes": unpack_bytes},
    }
    # the single-launch step moves what the three stages move, except that the attention output
    # goes straight to both destinations (o is not read back) and gather_idx is not re-read
    fused = (w.B * w.N + 2 * T * row + 4 * (w.B + 1) + 4 * T) + 4 * T * row + \
            (T * row if fill_mode == 0 else w.B * w.N * row)
    stages["pack_attn_unpack"] = {"bytes": fused, "flops": stages["attn"]["flops"]}
    return stages


def capture(torch, fn, reps: int = 1):
    """Record `reps` calls of fn into one HIP graph (side stream, torch's capture plumbing)."""
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        fn()                                          # warm the code path outside capture
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=s):
            for _ in range(reps):
                fn()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()
    return g


def event_samples_us(torch, launch, iters: int, warmup: int = 5):
    """GPU time of launch() in microseconds, one sample per call, HIP events on the launching stream."""
    for _ in range(warmup):
        launch()
    torch.cuda.synchronize()
    samples = []
    for _ in range(iters):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        launch()
        e1.record()
        e1.synchronize()
        samples.append(e0.elapsed_time(e1) * 1e3)
    return samples


def event_time_us(torch, launch, iters: int, warmup: int = 5):
    """Median / mean GPU time of launch() in microseconds."""
    samples = event_samples_us(torch, launch, iters, warmup)
    return statistics.median(samples), statistics.fmean(samples)


def kernel_time_us(torch, fn, iters: int = 50, reps: int = REPLICAS):
    """One kernel alone: `reps` back-to-back copies of fn() in one HIP graph, HIP events around each of `iters`
    replays; spread() of the per-copy times in microseconds (includes the in-graph kernel-to-kernel gap)."""
    g = capture(torch, fn, reps)
    return spread([t / reps for t in event_samples_us(torch, g.replay, iters)])


def pick_streams(torch, n: int, bind, extra: int = 3, burst: int = 300):
    """n HIP streams (default priority) whose work overlaps, and the step function bound to them.
    HIP streams share a small number of hardware queues (four per process here) and two streams behind one
    queue run their kernels one after the other; which streams share is not visible from the API (a burst
    of empty kernels does not tell them apart either).  So a few more streams than needed are drawn,
    `bind(selection)` -- which returns a function that issues one step of the caller's real work on the
    given streams, round-robin -- is timed over a short burst for several selections of n, and the
    fastest selection is kept.  Returns (streams, step)."""
    pool = [torch.cuda.Stream() for _ in range(n + extra)]
    for st in pool:
        st.wait_stream(torch.cuda.current_stream())
    selections = [pool[i:i + n] for i in range(len(pool) - n + 1)]
    if extra > 0 and len(pool) >= 2 * n:
        selections.append(pool[::2][:n])
    best = None
    for sel in selections:
        step = bind(sel)
        if len(selections) == 1:
            return sel, step
        for _ in range(max(10, burst // 5)):
            step()
        t = min(wall_steps(torch, step, burst) for _ in range(2))
        if best is None or t < best[0]:
            best = (t, sel, step)
    return best[1], best[2]


class StreamedSteps:
    """Independent steps in flight on several HIP streams (default priority, chosen by pick_streams): one set
    of device buffers and one pre-marshalled ragged_pack_attn_unpack call per stream, issued round-robin.
    A step is latency-bound (a 6 us kernel on a chip it cannot fill), so steps of different batches
    overlap on the GPU; every step still produces all of its outputs in its own buffers."""

    def __init__(self, w, fill_mode: int = 0, streams: int = 3, tune: bool = True):
        import itertools
        import torch
        self.paths = [Path(w, fill_mode) for _ in range(streams)]

        def bind(selection):
            calls = []
            for st, p in zip(selection, self.paths):
                with torch.cuda.stream(st):
                    calls.append(p.prepared_one_launch())
            nxt = itertools.cycle(calls).__next__

            def step():                                # as little host work per step as Python allows
                nxt()()
            return step
        self.streams, self.step = pick_streams(torch, streams, bind, extra=3 if tune else 0)


def wall_steps(torch, fn, steps: int):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


class PaddedPath:
    """One attention layer on the padded layout: Q, K, V, O are [B, N, H, D] and the keep mask is
    applied inside the single ragged_attn_padded launch."""

    def __init__(self, w, fill_mode: int = 0):
        import torch
        from paper_2604_15408_amd import binding
        self.torch, self.b, self.w, self.fill_mode = torch, binding, w, fill_mode
        dev = "cuda:0"
        g = torch.Generator().manual_seed(w.seed * 7919 + 3)
        tdt = torch.float16 if w.dtype == "f16" else torch.bfloat16
        self.q, self.k, self.v = (torch.randn(w.B, w.N, w.H, w.D, generator=g, dtype=torch.float32)
                                  .to(tdt).to(dev) for _ in range(3))
        self.o = torch.zeros_like(self.q)
        self.keep = w.keep.to(dev)
        torch.cuda.synchronize()

    def run(self):
        self.b.ragged_attn_padded(self.q, self.k, self.v, self.o, self.keep, self.w.scale, self.fill_mode)

    def prepared(self):
        return self.b.prepare_attn_padded(self.q, self.k, self.v, self.o, self.keep, self.w.scale,
                                          self.fill_mode)


class Pipeline:
    """The 12-layer progressive-pruning loop (B=64, N=197, C=768): per layer
    pack(X_l, mask_l) -> ragged_attn(Q_l, K_l, V_l; cu_seqlens from pack) -> unpack(O_l) -> X_{l+1}.
    There are no projection weights, so Q/K/V of every layer are seeded N(0,1) tensors of that
    layer's packed length; pack's row output is produced (and parity-checked in the tests) but feeds
    nothing downstream.  All 36 launches use upper-bound grids, so the loop is graph-capturable.
    one_launch=True issues every layer as ONE ragged_pack_attn_unpack launch instead (12 kernels, the same
    outputs bit for bit); its Q/K/V/O buffers then hold B*N rows, as that entry point asks."""

    def __init__(self, layers, fill_mode: int = 1, one_launch: bool = False):
        import torch
        from paper_2604_15408_amd import binding
        self.torch, self.b, self.layers, self.fill_mode, self.one_launch = torch, binding, layers, fill_mode, one_launch
        dev = "cuda:0"
        w0 = layers[0]
        B, N, C, H, D = w0.B, w0.N, w0.C, w0.H, w0.D
        self.x = [w0.features().to(dev)] + [torch.zeros(B, N, C, dtype=torch.float16, device=dev)
                                            for _ in layers]
        self.keep = [w.keep.to(dev) for w in layers]
        self.packed = torch.zeros(B * N, C, dtype=torch.float16, device=dev)
        self.cu = [torch.zeros(B + 1, dtype=torch.int32, device=dev) for _ in layers]
        self.gidx = [torch.zeros(B * N, dtype=torch.int32, device=dev) for _ in layers]
        rows = lambda w: B * N if one_launch else max(w.T, 1)
        self.qkv = []
        for w in layers:
            bufs = tuple(torch.zeros(rows(w), H, D, dtype=torch.float16, device=dev) for _ in range(3))
            for dst, src in zip(bufs, w.qkv(max(w.T, 1))):
                dst[: src.shape[0]] = src.to(dev)              # rows past T are never read
            self.qkv.append(bufs)
        self.o = [torch.zeros(rows(w), H, D, dtype=torch.float16, device=dev) for w in layers]
        self.launches = (1 if one_launch else 3) * len(layers)
        torch.cuda.synchronize()

    def run(self):
        b = self.b
        for l, w in enumerate(self.layers):
            q, k, v = self.qkv[l]
            if self.one_launch:
                b.ragged_pack_attn_unpack(self.x[l], self.keep[l], q, k, v, self.packed, self.cu[l], self.gidx[l],
                                          self.o[l], self.x[l + 1], w.scale, self.fill_mode)
                continue
            b.ragged_pack(self.x[l], self.keep[l], self.packed, self.cu[l], self.gidx[l])
            b.ragged_attn(q, k, v, self.o[l], self.cu[l], w.N, w.scale)
            b.ragged_unpack(self.o[l].view(-1, w.C), self.keep[l], self.cu[l], self.gidx[l],
                            self.x[l + 1], self.fill_mode)

    @property
    def tokens(self) -> int:
        return sum(w.T for w in self.layers)


class StayPackedPipeline:
    """The same 12 layers kept in the packed layout throughout (the paper's Section 4.3 flow): one
    ragged_pack in front, per layer ragged_attn_strided on a fused [T_l, 3, H, D] QKV buffer, a
    ragged_repack where the schedule prunes again, and ragged_cls_extract at the end.  As in
    Pipeline there are no projection weights: each layer's QKV buffer is seeded data, and the
    attention output is the row tensor that the next re-pack prunes."""

    def __init__(self, layers):
        import torch
        from paper_2604_15408_amd import binding
        from paper_2604_15408_amd import workloads as wl
        self.torch, self.b, self.layers = torch, binding, layers
        dev = "cuda:0"
        w0 = layers[0]
        B, N, C, H, D = w0.B, w0.N, w0.C, w0.H, w0.D
        cap = B * N
        self.x = w0.features().to(dev)
        self.keep0 = w0.keep.to(dev)
        row_masks = wl.pipeline_row_masks([w.keep for w in layers])
        # a layer re-packs when its mask differs from the previous layer's
        self.prunes = [l for l in range(1, len(layers)) if not bool(row_masks[l].all())]
        self.row_keep = {l: torch.nn.functional.pad(row_masks[l], (0, cap - row_masks[l].numel())).to(dev)
                         for l in self.prunes}
        self.rows = [torch.zeros(cap, C, dtype=torch.float16, device=dev) for _ in range(2)]
        self.cu = [torch.zeros(B + 1, dtype=torch.int32, device=dev) for _ in range(len(self.prunes) + 1)]
        self.gidx = [torch.zeros(cap, dtype=torch.int32, device=dev) for _ in range(len(self.prunes) + 1)]
        self.qkv = []
        for w in layers:
            q, k, v = w.qkv(max(w.T, 1))
            self.qkv.append(torch.stack((q, k, v), dim=1).contiguous().to(dev))      # [T_l, 3, H, D]
        self.o = [torch.zeros(max(w.T, 1), H, D, dtype=torch.float16, device=dev) for w in layers]
        self.cls = torch.zeros(B, C, dtype=torch.float16, device=dev)
        self.launches = 1 + len(layers) + len(self.prunes) + 1
        torch.cuda.synchronize()

    def run(self):
        b, layers = self.b, self.layers
        b.ragged_pack(self.x, self.keep0, self.rows[0], self.cu[0], self.gidx[0])
        stage, cur = 0, 0
        for l, w in enumerate(layers):
            if l in self.prunes:
                # the previous layer's output rows are pruned again, packed to packed
                src = self.o[l - 1].view(-1, w.C)
                b.ragged_repack(src, self.row_keep[l][: src.shape[0]], self.cu[stage], self.rows[1 - cur],
                                self.cu[stage + 1], self.gidx[stage + 1])
                stage, cur = stage + 1, 1 - cur
            qkv = self.qkv[l]
            b.ragged_attn_strided(qkv[:, 0], qkv[:, 1], qkv[:, 2], self.o[l], self.cu[stage], w.N, w.scale)
        b.ragged_cls_extract(self.o[-1].view(-1, layers[-1].C), self.cu[stage], self.cls)

    @property
    def tokens(self) -> int:
        return sum(w.T for w in self.layers)


LN_EPS = 1e-6                    # LayerNorm epsilon of ViT / DeiT encoders


class PackedBlocks:
    """`depth` pre-norm encoder blocks run entirely on the packed buffer (the paper's Section 4.3 item
    4, "late blocks"): one ragged_pack in front, then per block
        h = LN(x); qkv = h Wqkv^T + b; a = ragged_attn_strided(qkv); x = x + a Wo^T + b;
        h = LN(x); x = x + GELU(h W1^T + b1) W2^T + b2
    (7 launches), and ragged_cls_extract at the end.  Weights are seeded synthetic tensors; every
    launch takes the packed row count from cu_seqlens[B] on the device, so the loop is capturable
    and its cost follows the number of kept tokens."""

    def __init__(self, w, depth: int = 8, shared_weights: bool = True, rows_cap: int | None = None,
                 rows_hint: int = 0):
        """rows_cap: row capacity of the packed buffers.  B*N always works; a pruning method that keeps a
        fixed number of tokens per image knows T on the host and can pass it, which lets the linear
        layers size their grids for the real row count.  rows_hint: the expected number of kept rows
        (keep ratio * B * N) when only that is known; the linear layers pick their tile shape from it."""
        import torch
        from paper_2604_15408_amd import binding
        from paper_2604_15408_amd import workloads as wl
        self.torch, self.b, self.w, self.depth = torch, binding, w, depth
        dev = "cuda:0"
        B, N, C, H, D = w.B, w.N, w.C, w.H, w.D
        cap = B * N if rows_cap is None else int(rows_cap)
        if cap < w.T:
            raise ValueError("rows_cap is smaller than the number of kept tokens")
        self.cap, self.hidden, self.rows_hint = cap, 4 * C, int(rows_hint)
        tdt = torch.float16 if w.dtype == "f16" else torch.bfloat16
        self.x_in = w.features().to(dev)
        self.keep = w.keep.to(dev)
        self.cu = torch.zeros(B + 1, dtype=torch.int32, device=dev)
        self.gidx = torch.zeros(cap, dtype=torch.int32, device=dev)
        self.rows = self.cu[B:]                                     # device row count T
        sets = 1 if shared_weights else depth
        self.params = [{k: v.to(dev) for k, v in wl.block_weights(C, 4 * C, w.dtype, 2000 + i).items()}
                       for i in range(sets)]
        z = lambda *shape: torch.zeros(*shape, dtype=tdt, device=dev)
        self.x, self.h, self.qkv, self.a, self.mid = z(cap, C), z(cap, C), z(cap, 3, H, D), z(cap, H, D), z(cap, 4 * C)
        self.cls = z(B, C)
        self.launches = 1 + 7 * depth + 1
        torch.cuda.synchronize()

    def block(self, p):
        b, w, rows, hint = self.b, self.w, self.rows, self.rows_hint
        C = w.C
        b.ragged_layernorm(self.x, p["ln1_g"], p["ln1_b"], self.h, rows, LN_EPS)
        b.ragged_linear(self.h, p["w_qkv"], p["b_qkv"], None, self.qkv.view(self.cap, 3 * C), rows, rows_hint=hint)
        b.ragged_attn_strided(self.qkv[:, 0], self.qkv[:, 1], self.qkv[:, 2], self.a, self.cu, w.N, w.scale)
        b.ragged_linear(self.a.view(self.cap, C), p["w_o"], p["b_o"], self.x, self.x, rows, rows_hint=hint)
        b.ragged_layernorm(self.x, p["ln2_g"], p["ln2_b"], self.h, rows, LN_EPS)
        b.ragged_linear(self.h, p["w_fc1"], p["b_fc1"], None, self.mid, rows, "gelu", rows_hint=hint)
        b.ragged_linear(self.mid, p["w_fc2"], p["b_fc2"], self.x, self.x, rows, rows_hint=hint)

    def run(self):
        self.b.ragged_pack(self.x_in, self.keep, self.x, self.cu, self.gidx)
        for i in range(self.depth):
            self.block(self.params[i % len(self.params)])
        self.b.ragged_cls_extract(self.x, self.cu, self.cls)

    def flops(self) -> int:
        w, T = self.w, self.w.T
        C = w.C
        linear = 2 * T * (3 * C * C + C * C + 2 * C * self.hidden)
        attn = 4 * w.D * w.H * sum(n * n for n in w.lengths)
        return self.depth * (linear + attn)


class ProgressiveBlocks:
    """The whole flow of the paper's Section 4.3 with real blocks: a `depth`-block pre-norm encoder (synthetic
    weights) that prunes tokens in front of the blocks listed in `prune_at` and never leaves the packed
    layout.  A pruning stage is three launches -- ragged_token_scores_l2 on the packed rows,
    ragged_keep_topk (class token plus the k - 1 best others per image, k = round(keep_ratio * n)) and
    ragged_repack -- so every image keeps the same, host-known number of tokens and each stage's buffers
    have exactly B * n_s rows; blocks are the seven launches of PackedBlocks; ragged_cls_extract ends the
    run.  Everything is device-side and capturable in one HIP graph."""

    def __init__(self, B: int, N: int = 197, H: int = 12, D: int = 64, depth: int = 12, prune_at=(3, 6, 9),
                 keep_ratio: float = 0.7, dtype: str = "f16", seed: int = 3000, shared_weights: bool = True):
        import torch
        from paper_2604_15408_amd import binding
        from paper_2604_15408_amd import workloads as wl
        self.torch, self.b = torch, binding
        self.B, self.N, self.H, self.D, self.depth = B, N, H, D, depth
        self.C = C = H * D
        self.scale = D ** -0.5
        self.prune_at = tuple(sorted(prune_at))
        dev = "cuda:0"
        tdt = torch.float16 if dtype == "f16" else torch.bfloat16
        self.lengths = [N]                                     # tokens per image at every stage
        for _ in self.prune_at:
            self.lengths.append(max(1, int(round(keep_ratio * self.lengths[-1]))))
        keep_all = torch.ones(B, N, dtype=torch.uint8)
        self.input = wl.Workload("progressive_input", B, N, H, D, dtype, seed, keep_all)
        self.x_in = self.input.features().to(dev)
        self.keep_all = keep_all.to(dev)
        z = lambda *shape, dt=tdt: torch.zeros(*shape, dtype=dt, device=dev)
        self.x = [z(B * n, C) for n in self.lengths]           # packed activations of every stage
        self.cu = [z(B + 1, dt=torch.int32) for _ in self.lengths]
        self.gidx = [z(B * n, dt=torch.int32) for n in self.lengths]
        self.scores = [z(B, n, dt=torch.float64) for n in self.lengths[:-1]]
        self.keep = [z(B, n, dt=torch.uint8) for n in self.lengths[:-1]]
        rows0 = B * N
        self.h, self.qkv, self.a, self.mid = z(rows0, C), z(rows0, 3, H, D), z(rows0, H, D), z(rows0, 4 * C)
        self.cls = z(B, C)
        sets = 1 if shared_weights else depth
        self.params = [{k: v.to(dev) for k, v in wl.block_weights(C, 4 * C, dtype, seed + 1 + i).items()}
                       for i in range(sets)]
        self.launches = 1 + 7 * depth + 3 * len(self.prune_at) + 1
        self.stage = 0
        torch.cuda.synchronize()

    def pack_all(self):
        self.stage = 0
        self.b.ragged_pack(self.x_in, self.keep_all, self.x[0], self.cu[0], self.gidx[0])

    def prune(self):
        """scores -> top-k keep mask -> re-pack; moves on to the next stage's buffers."""
        b, s = self.b, self.stage
        n, k = self.lengths[s], self.lengths[s + 1]
        b.ragged_token_scores_l2(self.x[s].view(self.B, n, self.C), self.scores[s])
        b.ragged_keep_topk(self.scores[s], k, self.keep[s])
        b.ragged_repack(self.x[s], self.keep[s].view(-1), self.cu[s], self.x[s + 1], self.cu[s + 1], self.gidx[s + 1])
        self.stage = s + 1

    def block(self, p):
        b, s, C = self.b, self.stage, self.C
        rows = self.B * self.lengths[s]
        x, cu = self.x[s], self.cu[s]
        rows_dev = cu[self.B:]
        h, qkv, a, mid = self.h[:rows], self.qkv[:rows], self.a[:rows], self.mid[:rows]
        b.ragged_layernorm(x, p["ln1_g"], p["ln1_b"], h, rows_dev, LN_EPS)
        b.ragged_linear(h, p["w_qkv"], p["b_qkv"], None, qkv.view(rows, 3 * C), rows_dev)
        b.ragged_attn_strided(qkv[:, 0], qkv[:, 1], qkv[:, 2], a, cu, self.lengths[s], self.scale)
        b.ragged_linear(a.view(rows, C), p["w_o"], p["b_o"], x, x, rows_dev)
        b.ragged_layernorm(x, p["ln2_g"], p["ln2_b"], h, rows_dev, LN_EPS)
        b.ragged_linear(h, p["w_fc1"], p["b_fc1"], None, mid, rows_dev, "gelu")
        b.ragged_linear(mid, p["w_fc2"], p["b_fc2"], x, x, rows_dev)

    def run(self):
        self.pack_all()
        for blk in range(self.depth):
            if blk in self.prune_at:
                self.prune()
            self.block(self.params[blk % len(self.params)])
        self.b.ragged_cls_extract(self.x[self.stage], self.cu[self.stage], self.cls)

    def tokens(self) -> int:
        """Token-blocks processed in one run (rows summed over the blocks)."""
        total, s = 0, 0
        for blk in range(self.depth):
            if blk in self.prune_at:
                s += 1
            total += self.B * self.lengths[s]
        return total


class Ceilings:
    """What this GPU actually reaches on the two resources the rooflines are drawn against: a streaming read
    and a streaming copy of 1 GiB (HBM) and a register-resident fp16 MFMA loop (matrix cores).  The kernels
    live in the benchmark's own shared library (native/ceilings.hip), not in the C ABI."""

    def __init__(self):
        import ctypes
        from pathlib import Path as FsPath
        path = FsPath(__file__).resolve().parent / "libragged_ceilings.so"
        if not path.exists():
            raise FileNotFoundError(f"{path} is missing: build it with `python -m paper_2604_15408_amd.build`")
        lib = ctypes.CDLL(str(path))
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        lib.ceiling_stream_read.argtypes = [vp, i64, vp, i32, i32, vp]
        lib.ceiling_stream_copy.argtypes = [vp, vp, i64, i32, i32, vp]
        lib.ceiling_mfma_loop.argtypes = [i32, i32, vp, vp]
        lib.ceiling_mfma_flops.argtypes = [i32, i32]
        lib.ceiling_mfma_flops.restype = i64
        self.lib = lib

    def measure(self, torch, gib: float = 1.0, iters: int = 8):
        """Best rate over a few launch shapes (1, 2, 4 and 8 work-groups per CU; plain and non-temporal
        accesses): the rates differ by 20-30 % between shapes on this part, and a ceiling is the best of them."""
        lib = self.lib
        words = int(gib * (1 << 30)) // 4
        src = torch.full((words,), 0x01010101, dtype=torch.int32, device="cuda:0")
        dst = torch.empty_like(src)
        sink = torch.zeros(1024, dtype=torch.int32, device="cuda:0")
        nbytes = words * 4
        stream = lambda: torch.cuda.current_stream().cuda_stream

        def check(rc):
            if rc != 0:
                raise RuntimeError(f"ceiling kernel launch failed with hipError {rc}")

        def best(launch):
            found = None
            for groups in (256, 512, 1024, 2048):
                for nt in (0, 1):
                    us = spread(event_samples_us(torch, lambda: check(launch(groups, nt)), iters, warmup=2))["median"]
                    if found is None or us < found[0]:
                        found = (us, groups, nt)
            return found
        r_us, r_groups, r_nt = best(lambda g, nt: lib.ceiling_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), g, nt, stream()))
        c_us, c_groups, c_nt = best(lambda g, nt: lib.ceiling_stream_copy(src.data_ptr(), dst.data_ptr(), nbytes, g, nt, stream()))
        mfma = {}
        for label, mfma_iters in (("burst", 100), ("sustained", 2000)):          # ~0.1 ms and ~1.5 ms per launch
            groups = 256 * 8                                                     # eight wavefronts per SIMD
            us = spread(event_samples_us(
                torch, lambda: check(lib.ceiling_mfma_loop(mfma_iters, groups, sink.data_ptr(), stream())), iters, warmup=2))["median"]
            mfma[label] = lib.ceiling_mfma_flops(mfma_iters, groups) / us / 1e6
        del src, dst
        return {"hbm_read_gbs": nbytes / r_us / 1e3, "hbm_read_shape": {"groups": r_groups, "nontemporal": bool(r_nt)},
                "hbm_copy_gbs": 2 * nbytes / c_us / 1e3, "hbm_copy_shape": {"groups": c_groups, "nontemporal": bool(c_nt)},
                "mfma_f16_tflops": mfma["sustained"], "mfma_f16_tflops_burst": mfma["burst"], "buffer_gib": gib,
                "note": "1 GiB streaming read / copy (copy counts read + written bytes) and a register-resident "
                        "v_mfma_f32_16x16x32_f16 loop (eight chains per wavefront, eight wavefronts per SIMD); HIP-event "
                        "medians; the MFMA rate is limited by the clock the chip holds under that load"}


class ColdSets:
    """`sets` copies of every buffer of a workload, launched one after the other inside one graph, so that by
    the time a copy comes round again the others have pushed it out of the L2s and the 256 MB Infinity Cache."""

    def __init__(self, w, sets: int, fill_mode: int = 0):
        self.paths = [Path(w, fill_mode) for _ in range(sets)]
        self.sets = sets

    def time_us(self, torch, what: str = "one_launch", iters: int = 20):
        def all_sets():
            for p in self.paths:
                getattr(p, what)()
        all_sets()
        torch.cuda.synchronize()
        g = capture(torch, all_sets)
        return spread([t / self.sets for t in event_samples_us(torch, g.replay, iters)])


def config_point(torch, w, steps: int = 200, blocks: int = 7):
    """Compact record of one benchmark configuration: ragged_attn alone and the whole step in one launch
    (kernel time inside a graph, HBM fraction of the algorithmic bytes), and the wall-clock step on one stream."""
    p = Path(w, 0)
    p.pack()                                          # cu_seqlens for the attention launches below
    torch.cuda.synchronize()
    alg = p.algorithmic()
    attn = kernel_time_us(torch, p.attn, iters=20)
    step = kernel_time_us(torch, p.one_launch, iters=20)
    wall = wall_blocks(torch, p.prepared_one_launch(), steps, blocks)
    frac = lambda name, us: alg[name]["bytes"] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS
    return {"workload": w.name, "dtype": w.dtype, "B": w.B, "N": w.N, "T": w.T, "max_len": max(w.lengths),
            "attn_us": attn["median"], "attn_hbm_frac": frac("attn", attn["median"]),
            "attn_tflops": alg["attn"]["flops"] / attn["median"] / 1e6,
            "step_kernel_us": step["median"], "step_hbm_frac": frac("pack_attn_unpack", step["median"]),
            "step_wall_us": wall["median"] * 1e6, "step_tokens_per_s": w.T / wall["median"]}


def pipeline_point(torch, pipe, kernels: int, alg_bytes: int | None = None):
    """A whole multi-layer loop captured in one HIP graph: GPU time of a replay, wall-clock per replay, tokens/s."""
    pipe.run()
    torch.cuda.synchronize()
    g = capture(torch, pipe.run)
    gpu = spread(event_samples_us(torch, g.replay, 30))
    wall = spread([wall_steps(torch, g.replay, 50) for _ in range(7)])
    rec = {"kernels_in_graph": kernels, "tokens": pipe.tokens, "graph_gpu_us": gpu["median"],
           "graph_gpu_us_p10_p90": [gpu["p10"], gpu["p90"]], "graph_wall_us": wall["median"] * 1e6,
           "tokens_per_s": pipe.tokens / wall["median"]}
    if alg_bytes:
        rec["hbm_frac"] = alg_bytes / (gpu["median"] * 1e-6) / 1e9 / HBM_PEAK_GBS
    return rec
