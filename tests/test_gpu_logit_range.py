"""GPU parity on inputs whose logits span tens of natural units and grow (or fall, or jump)
along the pattern: the attention kernels keep their softmax reference until a tile's weights
outgrow it, so these are the inputs on which the reference has to be raised again and again,
by large steps, in the scheduled steps, in the first and last half-steps, and in the ragged last
tile.  Ordinary N(0,1) inputs raise it rarely or never."""

import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2605_20813_amd import pulsecol as pc
from parity_util import assert_close, f64, random_idx

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def steep_qkv(B, H, n, d, dtype, seed, shape, span):
    """Q, K, V whose logits q_i.k_j/sqrt(d) are ~ span * ramp_j (+ noise of order 1): component 0
    of every query is about 1, component 0 of key j carries the ramp.  `shape`: "up" (grows with
    the column number: every tile outgrows the reference), "down" (the first tile holds the
    maximum), "late" (flat, then a jump in the last few columns: the ragged last tile raises it),
    "saw" (rises and collapses every 200 columns)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    Q = torch.randn(B, H, n, d, generator=g) * 0.3
    K = torch.randn(B, H, n, d, generator=g) * 0.3
    V = torch.randn(B, H, n, d, generator=g)
    Q[..., 0] = 1.0 + 0.2 * torch.randn(B, H, n, generator=g)
    t = torch.arange(n, dtype=torch.float32) / max(1, n - 1)
    ramp = {"up": t, "down": 1.0 - t, "late": (t > 0.995).float(), "saw": (torch.arange(n) % 200).float() / 200.0}[shape]
    K[..., 0] = ramp * (span * d ** 0.5)
    return Q.to(dtype), K.to(dtype), V.to(dtype)


def kind_of(dtype):
    return "bf16" if dtype == torch.bfloat16 else "f32"


@pytest.mark.parametrize("shape", ["up", "down", "late", "saw"])
@pytest.mark.parametrize("n,d,dtype,G,k,span", [
    (1500, 128, torch.bfloat16, 0, 1100, 60.0),     # main kernel, 18 tiles, ragged last tile
    (1500, 128, torch.bfloat16, 0, 1500, 25.0),     # keep everything (idx = a permutation-free full set)
    (900, 64, torch.bfloat16, 0, 700, 40.0),        # head dimension 64
    (1200, 128, torch.bfloat16, 128, 1000, 60.0),   # small-group kernel, 4 waves
    (700, 128, torch.bfloat16, 64, 650, 40.0),      # 2 waves
    (500, 64, torch.bfloat16, 32, 470, 40.0),       # 1 wave, head dimension 64
    # fp32 kernels: a smaller span, since the rounding of a dot product of magnitude span*sqrt(d)
    # in fp32 is an error of the logit itself (1e-4 of the weights at span 60)
    (600, 128, torch.float32, 0, 500, 25.0),
])
def test_sparse_attention_with_steep_logits(shape, n, d, dtype, G, k, span):
    B, H = 1, 2
    say(f"steep attn case {shape} n={n} d={d} {dtype} G={G} k={k} span={span}")
    Q, K, V = steep_qkv(B, H, n, d, dtype, seed=n + k + len(shape), shape=shape, span=span)
    U = 1 if G == 0 else -(-n // G)
    idx = random_idx(n, k, B * H * U, seed=7 * n + k).view(B, H, U, k)
    with pc.Context(B, H, n, d, dtype, group_size=G) as ctx:
        O = ctx.attn(Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV))
        torch.cuda.synchronize()
    for h in range(H):
        q, k_, v = f64(Q[0, h]), f64(K[0, h]), f64(V[0, h])
        for u in range(U):
            lo, hi = (0, n) if G == 0 else (u * G, min(n, (u + 1) * G))
            want = oracle.sparse_attention_masked(q[lo:hi], k_, v, idx[0, h, u].numpy())
            assert_close(O[0, h, lo:hi], want, kind_of(dtype), f"steep {shape} h{h} group {u}")


@pytest.mark.parametrize("shape", ["up", "down", "late", "saw"])
@pytest.mark.parametrize("n,d,dtype,span", [(1300, 128, torch.bfloat16, 60.0), (700, 64, torch.bfloat16, 40.0),
                                            (400, 128, torch.float32, 25.0)])
def test_dense_attention_and_lse_with_steep_logits(shape, n, d, dtype, span):
    B, H = 1, 2
    say(f"steep dense case {shape} n={n} d={d} {dtype} span={span}")
    Q, K, V = steep_qkv(B, H, n, d, dtype, seed=3 * n + len(shape), shape=shape, span=span)
    with pc.Context(B, H, n, d, dtype) as ctx:
        lse = torch.empty(B, H, n, dtype=torch.float32, device=DEV)
        O = ctx.attn_dense(Q.to(DEV), K.to(DEV), V.to(DEV), lse_out=lse)
        torch.cuda.synchronize()
    for h in range(H):
        q, k_, v = f64(Q[0, h]), f64(K[0, h]), f64(V[0, h])
        assert_close(O[0, h], oracle.dense_attention(q, k_, v), kind_of(dtype), f"steep dense {shape} h{h}")
        Z = oracle.attention_logits(q, k_)
        m = Z.max(axis=1)
        want_lse = m + np.log(np.exp(Z - m[:, None]).sum(axis=1))
        np.testing.assert_allclose(f64(lse[0, h]), want_lse, rtol=0, atol=2e-5 * max(1.0, np.abs(want_lse).max()))


@pytest.mark.parametrize("shape", ["up", "saw"])
@pytest.mark.parametrize("n,d,dtype", [(1100, 128, torch.bfloat16), (500, 64, torch.float32)])
def test_scores_with_steep_logits(shape, n, d, dtype):
    """The two select passes on the same inputs: the row pass raises its reference as above, the
    column pass takes exp2 of differences of tens of units.  Columns that carry next to no mass
    are compared in absolute terms (their relative error is that of exp of a large argument)."""
    B, H = 1, 2
    span = 40.0
    say(f"steep scores case {shape} n={n} d={d} {dtype}")
    Q, K, _ = steep_qkv(B, H, n, d, dtype, seed=5 * n + len(shape), shape=shape, span=span)
    with pc.Context(B, H, n, d, dtype) as ctx:
        s = ctx.scores(Q.to(DEV), K.to(DEV))
        torch.cuda.synchronize()
    for h in range(H):
        want = oracle.column_scores(f64(Q[0, h]), f64(K[0, h]))[0]
        got = f64(s[0, h, 0])
        assert abs(got.sum() - 1.0) < 1e-5
        # relative error of exp(z - lse) ~ absolute error of z - lse ~ 1e-6 * |z|
        assert np.abs(got - want).max() <= 2e-4 * want.max()
        big = want > 1e-6 * want.max()
        assert (np.abs(got - want)[big] / want[big]).max() < 2e-4
