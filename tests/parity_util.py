"""Helpers shared by the GPU parity tests: tolerances of the acceptance bar and the
comparison rules for column sets."""

import numpy as np
import torch

import oracle

# acceptance bar: outputs within max-abs / mean-abs of the fp64 oracle
TOL = {
    "bf16": dict(max_abs=2e-2, mean_abs=2e-3),
    "f32": dict(max_abs=1e-4, mean_abs=1e-5),
}
NEAR_TIE_REL_GAP = 1e-6      # a differing column is accepted only within this relative score gap


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").double().numpy()


def assert_close(got: torch.Tensor, want: np.ndarray, kind: str, what: str = ""):
    g = f64(got)
    assert g.shape == want.shape, (g.shape, want.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    err = np.abs(g - want)
    tol = TOL[kind]
    assert err.max() <= tol["max_abs"], f"{what}: max abs err {err.max():.3e} > {tol['max_abs']}"
    assert err.mean() <= tol["mean_abs"], f"{what}: mean abs err {err.mean():.3e} > {tol['mean_abs']}"


def assert_idx_matches(got_idx: np.ndarray, scores64: np.ndarray, k: int, what: str = ""):
    """`got_idx` (one row, from the GPU) against the oracle's top-k of its OWN fp64 scores.

    Identical sets pass.  Otherwise every column the two sets disagree on must be a
    near-tie: its oracle score within NEAR_TIE_REL_GAP (relative) of the oracle's k-th
    largest score.  In all cases the GPU row must be k distinct ascending in-range columns.
    """
    n = scores64.shape[0]
    got = np.asarray(got_idx, dtype=np.int64)
    assert got.shape == (k,), what
    assert (got[1:] > got[:-1]).all(), f"{what}: not strictly ascending"
    assert got[0] >= 0 and got[-1] < n, f"{what}: out of range"
    want = oracle.topk_columns(scores64[None], k)[0]
    if np.array_equal(got, want):
        return 0
    kth = np.sort(scores64)[::-1][k - 1]
    diff = np.setxor1d(got, want)
    gaps = np.abs(scores64[diff] - kth) / kth
    assert gaps.max() <= NEAR_TIE_REL_GAP, \
        f"{what}: {diff.size} differing columns, worst relative gap {gaps.max():.3e} (allowed {NEAR_TIE_REL_GAP})"
    return int(diff.size)


def random_idx(n: int, k: int, rows: int, seed: int, sort: bool = True) -> torch.Tensor:
    """`rows` seeded random k-subsets of [0, n), int32 [rows, k] (no method arithmetic)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    out = torch.empty(rows, k, dtype=torch.int32)
    for r in range(rows):
        sel = torch.randperm(n, generator=g)[:k]
        out[r] = (torch.sort(sel).values if sort else sel).to(torch.int32)
    return out
