"""Refresh-schedule driver: which denoising steps re-identify the column pattern, for a stack
of attention layers that each keep their own cached pattern.

Orchestration only -- every computation is a call into the C-ABI library through
``pulsecol.Context``.  The schedule follows the paper's Sec. 3.3 (periodic refresh inside an
early window of floor(eta * T) steps, reuse everywhere else) and the placement variants of its
appendix ablation (uniform = default, power-based, random).
"""

from __future__ import annotations

from . import pulsecol as pc

KINDS = ("uniform", "power", "random")


def refresh_steps(T: int, eta: float, R: int, kind: str = "uniform", uniforms=None):
    """0-based refresh steps of a run of T denoising steps (the library returns 1-based)."""
    if kind == "uniform":
        tau = pc.refresh_schedule(T, eta, R)
    elif kind == "power":
        tau = pc.refresh_schedule_power(T, eta, R)
    elif kind == "random":
        if uniforms is None:
            raise ValueError("the random schedule needs R-1 uniforms in [0, 1)")
        tau = pc.refresh_schedule_random(T, eta, R, uniforms)
    else:
        raise ValueError(f"kind must be one of {KINDS}")
    return sorted({t - 1 for t in tau})


class LayerStack:
    """L layers of one shape; layer l owns context l and therefore its own cached pattern.

    ``step(t, qkv, out)`` runs one denoising step: at a refresh step every layer re-identifies
    its pattern from its current Q, K (``dense_at_refresh``: and returns the dense output of
    that step, as in the paper's description of the refresh step), at every other step it
    reuses the cached pattern in the column-sparse kernel.
    """

    def __init__(self, layers: int, batch: int, heads: int, seq: int, head_dim: int, dtype, keep_ratio: float,
                 steps_0based, group_size: int = 0, dense_at_refresh: bool = False, device: int = 0):
        if layers < 1:
            raise ValueError("layers must be >= 1")
        self.keep = keep_ratio
        self.refresh = frozenset(int(t) for t in steps_0based)
        if 0 not in self.refresh:
            raise ValueError("step 0 must identify the pattern")
        self.dense_at_refresh = dense_at_refresh
        self.ctx = [pc.Context(batch, heads, seq, head_dim, dtype, group_size=group_size, device=device,
                               max_keep_ratio=keep_ratio)
                    for _ in range(layers)]
        self.idx = [None] * layers

    def is_refresh(self, t: int) -> bool:
        return t in self.refresh

    def step(self, t: int, qkv, out):
        """qkv: per layer (Q, K, V); out: per layer O.  Returns the number of selects run."""
        selects = 0
        for l, ctx in enumerate(self.ctx):
            Q, K, V = qkv[l]
            if self.is_refresh(t):
                selects += 1
                if self.dense_at_refresh:
                    _, self.idx[l] = ctx.refresh_dense(Q, K, V, self.keep, O=out[l], idx_out=self.idx[l])
                    continue
                self.idx[l] = ctx.select(Q, K, self.keep, refresh=True, idx_out=self.idx[l])
            ctx.attn(Q, K, V, self.idx[l], O=out[l])
        return selects

    def close(self):
        for c in self.ctx:
            c.close()
        self.ctx = []

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
