"""Seeded synthetic inputs with the shapes of the LLaDA-style workloads.

This module only draws random numbers and rounds them to the storage type.  It
contains none of the method's arithmetic (no logits, softmax, scores, top-k or
keep-count rule), so that the GPU path and the CPU checker can both take their
inputs from it without sharing any computation.

Recipe (per head, generator seeded by (seed, batch index, head index)):
  Q, K, V ~ N(0, 1) in fp32; ``heavy`` distinct key positions drawn without
  replacement have their K rows multiplied by ``heavy_scale`` in fp32; the
  result is rounded to the storage dtype (bf16 or fp32).  Drift steps add
  ``sigma * N(0, 1)`` to fp32 master copies and round again.
"""

from __future__ import annotations

from dataclasses import dataclass, field

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    heads: int
    seq: int
    head_dim: int
    dtype: str              # "bf16" | "f32"
    keep_ratios: tuple      # kept fraction(s) of key columns, 1 - sparsity
    heavy: int              # planted heavy key columns per head
    heavy_scale: float
    seed: int
    steps: int = 1                       # denoising steps in the schedule
    refresh_steps: tuple = (0,)          # 0-based steps at which the pattern is (re)selected
    drift_sigma: float = 0.0
    note: str = field(default="", compare=False)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


WORKLOADS = {
    "tiny": Workload("tiny", 1, 2, 256, 64, "f32", (0.25,), 16, 3.0, 20813,
                     steps=1, refresh_steps=(0,),
                     note="one select + one attn; the CPU checker finishes in well under a second"),
    "llada_4k": Workload("llada_4k", 1, 32, 4096, 128, "bf16", (0.10,), 204, 2.5, 20814,
                         steps=8, refresh_steps=(0,),
                         note="select at step 0, then 8 attn steps reusing the indices"),
    "llada_16k": Workload("llada_16k", 1, 32, 16384, 128, "bf16", (0.10,), 819, 2.5, 20815,
                          steps=64, refresh_steps=(0, 16, 32), drift_sigma=0.05,
                          note="64 steps, select at 0/16/32, inputs drift between steps"),
    "llada_32k": Workload("llada_32k", 1, 32, 32768, 128, "bf16", (0.05, 0.10, 0.20), 1638, 2.5, 20816,
                          steps=1, refresh_steps=(0,),
                          note="keep-ratio sweep with a dense baseline at the same shape"),
    "llada_64k": Workload("llada_64k", 1, 32, 65536, 128, "bf16", (0.10,), 3276, 2.5, 20817,
                          steps=1024, refresh_steps=(0, 102, 204, 306),
                          note="1024 steps with 4 refreshes in the first 30% of steps"),
    # beyond the listed configurations: the longest context of the paper's kernel-speed figure, on a
    # quarter of the heads (timing and parity only)
    "llada_128k_8h": Workload("llada_128k_8h", 1, 8, 131072, 128, "bf16", (0.10,), 6553, 2.5, 20818,
                              steps=1, refresh_steps=(0,),
                              note="128K context, 8 of the 32 heads"),
}


def _gen(w: Workload, b: int, h: int, stream: int = 0) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(((w.seed * 1009 + b) * 1009 + h) * 17 + stream)
    return g


def heavy_columns(w: Workload, b: int, h: int) -> torch.Tensor:
    """The planted heavy key positions of one head (int64, ascending)."""
    g = _gen(w, b, h, stream=1)
    perm = torch.randperm(w.seq, generator=g)
    return torch.sort(perm[: w.heavy]).values


def make_head_fp32(w: Workload, b: int, h: int):
    """fp32 master copies (Q, K, V), each [seq, head_dim], heavy rows already scaled."""
    g = _gen(w, b, h, stream=0)
    q = torch.randn(w.seq, w.head_dim, generator=g, dtype=torch.float32)
    k = torch.randn(w.seq, w.head_dim, generator=g, dtype=torch.float32)
    v = torch.randn(w.seq, w.head_dim, generator=g, dtype=torch.float32)
    k[heavy_columns(w, b, h)] *= w.heavy_scale
    return q, k, v


def make_head(w: Workload, b: int, h: int):
    """(Q, K, V) of one head in the workload's storage dtype, on the CPU."""
    return tuple(t.to(w.torch_dtype) for t in make_head_fp32(w, b, h))


def make_qkv(w: Workload, heads=None, master: bool = False):
    """Packed [B, H', seq, head_dim] CPU tensors for the given head subset (default all).

    With ``master=True`` the fp32 master copies are returned instead of the
    rounded storage tensors (used by the drift schedule).
    """
    heads = list(range(w.heads)) if heads is None else list(heads)
    dt = torch.float32 if master else w.torch_dtype
    out = [torch.empty(w.batch, len(heads), w.seq, w.head_dim, dtype=dt) for _ in range(3)]
    for b in range(w.batch):
        for hi, h in enumerate(heads):
            for dst, src in zip(out, make_head_fp32(w, b, h)):
                dst[b, hi] = src.to(dt)
    return tuple(out)


def drift_(masters, w: Workload, step: int) -> None:
    """In place: X += sigma * N(0,1) on the fp32 master copies (seeded by the step).

    The noise is drawn on the device the masters live on (CPU and GPU generators give different
    streams: a run that wants identical buffers on both sides drifts on one and copies).
    """
    dev = masters[0].device
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed * 7919 + step)
    for x in masters:
        x.add_(torch.randn(x.shape, generator=g, dtype=torch.float32, device=dev), alpha=w.drift_sigma)


def random_scores(rows: int, n: int, seed: int, ties: bool = False) -> torch.Tensor:
    """fp32 [rows, n] positive values shaped like column scores (for top-k tests).

    With ``ties`` a quarter of the entries are overwritten by repeated values so
    that the selection threshold falls inside a run of equal scores.
    """
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    s = torch.rand(rows, n, generator=g, dtype=torch.float32) / n
    if ties:
        pick = torch.rand(rows, n, generator=g) < 0.25
        levels = torch.randint(1, 5, (rows, n), generator=g).to(torch.float32) / (4.0 * n)
        s = torch.where(pick, levels, s)
    return s
