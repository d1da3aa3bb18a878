"""Seeded synthetic inputs for the pack -> ragged attention -> unpack path.

This module holds NO arithmetic of the method (no prefix sums, no softmax, no gathers): it only
draws keep masks and N(0,1) tensors on the CPU from a seeded ``torch.Generator`` so that the HIP
path and the CPU oracle are fed the same bits on any machine.  Both sides may import it.

The paper's kernel measurements use synthetic N(0,1) tensors at DeiT-Base geometry (H=12, d=64,
197 tokens; Section 3.1 "Experimental Setup") with a fixed prune ratio; the high-resolution case
uses 577 tokens (Section 5.4).  The workloads below follow those shapes, with per-token Bernoulli
keep decisions so that the per-image lengths are ragged, and the CLS token (t = 0) always kept
(Section 4.3 item 5 reads CLS from the packed buffer).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np
import torch

_TORCH_DTYPE = {"f16": torch.float16, "bf16": torch.bfloat16}


@dataclass
class Workload:
    """One batch: geometry, dtype tag, seed and the keep mask (uint8 [B, N], CPU)."""
    name: str
    B: int
    N: int
    H: int
    D: int
    dtype: str                      # "f16" | "bf16"
    seed: int
    keep: torch.Tensor              # uint8 [B, N]
    scale: float = 0.125
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def C(self) -> int:
        return self.H * self.D

    @property
    def lengths(self) -> List[int]:
        return [int(v) for v in self.keep.to(torch.int64).sum(dim=1)]

    @property
    def T(self) -> int:
        return int(self.keep.to(torch.int64).sum())

    def features(self) -> torch.Tensor:
        """Token features x [B, N, C] ~ N(0,1), rounded to the workload dtype."""
        g = torch.Generator().manual_seed(self.seed * 7919 + 1)
        x = torch.randn(self.B, self.N, self.C, generator=g, dtype=torch.float32)
        return x.to(_TORCH_DTYPE[self.dtype])

    def qkv(self, rows: int | None = None):
        """Q, K, V [rows, H, D] ~ N(0,1) (rows defaults to the packed length T)."""
        rows = self.T if rows is None else rows
        g = torch.Generator().manual_seed(self.seed * 7919 + 2)
        out = []
        for _ in range(3):
            t = torch.randn(rows, self.H, self.D, generator=g, dtype=torch.float32)
            out.append(t.to(_TORCH_DTYPE[self.dtype]))
        return tuple(out)


def to_words(t: torch.Tensor) -> np.ndarray:
    """Reinterpret a CPU fp16/bf16 tensor as raw uint16 words (no value conversion)."""
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def keep_bernoulli(B: int, N: int, p, seed: int) -> torch.Tensor:
    """Per-token keep decisions: token t>0 of image i is kept with probability p (a float, or one
    value per image); token 0 (CLS) is always kept.  Lengths are 1 + Binomial(N-1, p_i)."""
    g = torch.Generator().manual_seed(seed)
    u = torch.rand(B, N, generator=g, dtype=torch.float64)
    p = torch.as_tensor(p, dtype=torch.float64).reshape(-1, 1)
    keep = (u < p).to(torch.uint8)
    keep[:, 0] = 1
    return keep


def keep_exact(N: int, counts: List[int], seed: int) -> torch.Tensor:
    """Masks with exactly counts[i] kept tokens: CLS (if counts[i] >= 1) plus a seeded random
    subset of the others.  counts[i] == 0 gives an all-dropped image (a degenerate case)."""
    g = torch.Generator().manual_seed(seed)
    B = len(counts)
    keep = torch.zeros(B, N, dtype=torch.uint8)
    for i, c in enumerate(counts):
        if not 0 <= c <= N:
            raise ValueError(f"count {c} outside [0, {N}]")
        perm = torch.randperm(N - 1, generator=g) + 1
        if c >= 1:
            keep[i, 0] = 1
            keep[i, perm[: c - 1]] = 1
    return keep


# ----------------------------------------------------------------------------------------------
# The five benchmark configurations (geometry and length recipe of each; seeds 1000 + index).
# ----------------------------------------------------------------------------------------------

def tiny(seed: int = 1000) -> Workload:
    """B=2, N=197, H=3, D=64 fp16; lengths exactly {197, 40} (DeiT-Ti head count)."""
    return Workload("tiny", 2, 197, 3, 64, "f16", seed, keep_exact(197, [197, 40], seed),
                    note="lengths {197, 40}")


def deit_b_pruned(keep_prob: float = 0.2, B: int = 32, dtype: str = "f16",
                  seed: int = 1001) -> Workload:
    """DeiT-Base attention geometry (N=197, H=12, D=64); per-image kept count is
    1 + Binomial(196, keep_prob) at uniformly random positions.  keep_prob=0.2 mirrors the
    80%-pruned rows of the paper's kernel-latency table."""
    keep = keep_bernoulli(B, 197, keep_prob, seed)
    return Workload(f"deit_b_keep{keep_prob:g}_bs{B}_{dtype}", B, 197, 12, 64, dtype, seed, keep,
                    note=f"1+Binomial(196,{keep_prob:g})")


def uniform(B: int, per_image: int, N: int = 197, dtype: str = "f16", seed: int = 1007) -> Workload:
    """Every image keeps exactly `per_image` tokens (class token + a seeded random subset): the
    uniform-length setting of the paper's kernel-latency tables (e.g. BS=32, 40 tokens per image)."""
    return Workload(f"uniform{per_image}_bs{B}_{dtype}", B, N, 12, 64, dtype, seed,
                    keep_exact(N, [per_image] * B, seed), note=f"exactly {per_image} per image")


SWEEP_KEEP_PROBS = (1.0, 0.8, 0.6, 0.4, 0.2, 0.1)


def sweep(seed: int = 1002) -> List[Workload]:
    """Pruning-ratio sweep at DeiT-Base shape in bf16."""
    return [deit_b_pruned(p, 32, "bf16", seed + 10 * k) for k, p in enumerate(SWEEP_KEEP_PROBS)]


def serving_384(B: int, seed: int = 1003) -> Workload:
    """384x384 inputs: N=577 (1 CLS + 24x24 patches), H=12, D=64 fp16; per-image keep probability
    drawn Uniform(0.2, 0.4), so lengths are ragged across the batch."""
    g = torch.Generator().manual_seed(seed + 17 * B)
    p = 0.2 + 0.2 * torch.rand(B, generator=g, dtype=torch.float64)
    keep = keep_bernoulli(B, 577, p, seed + 31 * B)
    return Workload(f"serving384_bs{B}", B, 577, 12, 64, "f16", seed + B, keep,
                    note="p_i~U(0.2,0.4), 1+Binomial(576,p_i)")


PIPELINE_PRUNE_LAYERS = (3, 6, 9)


def pipeline_masks(B: int = 64, N: int = 197, layers: int = 12, ratio: float = 0.7,
                   seed: int = 1004) -> List[torch.Tensor]:
    """Keep masks of a 12-layer progressive-pruning pipeline: all tokens kept in layers 1-2; at
    layers 3, 6 and 9 each surviving non-CLS token survives with probability ``ratio``."""
    g = torch.Generator().manual_seed(seed)
    keep = torch.ones(B, N, dtype=torch.uint8)
    masks = []
    for layer in range(1, layers + 1):
        if layer in PIPELINE_PRUNE_LAYERS:
            u = torch.rand(B, N, generator=g, dtype=torch.float64)
            keep = keep * (u < ratio).to(torch.uint8)
            keep[:, 0] = 1
        masks.append(keep.clone())
    return masks


def pipeline_row_masks(masks: List[torch.Tensor]) -> List[torch.Tensor]:
    """The same pruning schedule expressed on packed rows: entry l (l >= 1) holds one byte per row
    that survived masks[l-1], set if the row also survives masks[l] (pure indexing of the masks;
    entry 0 is masks[0] flattened, the first pack's own mask)."""
    rows = [masks[0].reshape(-1).clone()]
    for prev, cur in zip(masks[:-1], masks[1:]):
        rows.append(cur.reshape(-1)[prev.reshape(-1) != 0].clone())
    return rows


def pipeline(seed: int = 1004) -> List[Workload]:
    """One Workload per layer of the 12-layer pipeline (B=64, N=197, C=768, fp16)."""
    masks = pipeline_masks(seed=seed)
    return [Workload(f"pipeline_layer{l + 1}", 64, 197, 12, 64, "f16", seed + l + 1, m,
                     note="progressive keep 0.7 at layers 3/6/9")
            for l, m in enumerate(masks)]


def block_weights(C: int = 768, hidden: int = 3072, dtype: str = "f16", seed: int = 2000):
    """Seeded synthetic parameters of one pre-norm encoder block (there are no trained weights here):
    weights [out_features, in_features] ~ N(0, 1/in_features), biases ~ N(0, 0.02^2), LayerNorm gains
    1 + N(0, 0.1^2) and shifts N(0, 0.1^2).  Returned as CPU tensors of the activation dtype."""
    g = torch.Generator().manual_seed(seed)
    tdt = _TORCH_DTYPE[dtype]

    def rnd(*shape, scale=1.0, shift=0.0):
        return (torch.randn(*shape, generator=g, dtype=torch.float32) * scale + shift).to(tdt)

    return {
        "ln1_g": rnd(C, scale=0.1, shift=1.0), "ln1_b": rnd(C, scale=0.1),
        "w_qkv": rnd(3 * C, C, scale=C ** -0.5), "b_qkv": rnd(3 * C, scale=0.02),
        "w_o": rnd(C, C, scale=C ** -0.5), "b_o": rnd(C, scale=0.02),
        "ln2_g": rnd(C, scale=0.1, shift=1.0), "ln2_b": rnd(C, scale=0.1),
        "w_fc1": rnd(hidden, C, scale=C ** -0.5), "b_fc1": rnd(hidden, scale=0.02),
        "w_fc2": rnd(C, hidden, scale=hidden ** -0.5), "b_fc2": rnd(C, scale=0.02),
    }
