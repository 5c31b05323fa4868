"""Seeded sweep over irregular shapes: every kernel against the fp64 oracle at sizes chosen to
hit every remainder of the tile / pipeline structure (number of tiles modulo the unrolled
loop, ragged tails, ragged last groups, odd head counts)."""

import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2605_20813_amd import pulsecol as pc
from parity_util import assert_close, assert_idx_matches, f64, random_idx

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _cases():
    rng = np.random.default_rng(2605)
    out = []
    # the sparse kernel's steady loop runs (tiles - 2) iterations, unrolled by 4, tiles of 64 columns:
    # cover every remainder with exact and ragged tile counts, both head dims
    for tiles in range(1, 14):
        for ragged in (0, int(rng.integers(1, 64))):
            k = (tiles - 1) * 64 + (ragged if ragged else 64)
            n = int(k + rng.integers(0, 300))
            d = 128 if (tiles + (1 if ragged else 0)) % 3 else 64
            out.append((1, int(rng.integers(1, 4)), n, d, k))
    return out


@pytest.mark.parametrize("B,H,n,d,k", _cases())
def test_sparse_attention_every_tile_remainder(B, H, n, d, k):
    say(f"sweep attn B={B} H={H} n={n} d={d} k={k}")
    g = torch.Generator(device="cpu")
    g.manual_seed(n * 131 + k)
    Q, K, V = (torch.randn(B, H, n, d, generator=g).to(torch.bfloat16) for _ in range(3))
    idx = random_idx(n, k, B * H, seed=n + k).view(B, H, 1, k)
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx:
        O = ctx.attn(Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV))
        torch.cuda.synchronize()
    for h in range(H):
        want = oracle.sparse_attention_masked(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h]), idx[0, h].numpy())
        assert_close(O[0, h], want, "bf16", f"sweep attn n={n} k={k} head {h}")


@pytest.mark.parametrize("seed", range(8))
def test_random_configuration(seed):
    rng = np.random.default_rng(9000 + seed)
    d = int(rng.choice([64, 128]))
    H = int(rng.integers(1, 10))
    Hkv = int(rng.choice([x for x in range(1, H + 1) if H % x == 0]))
    n = int(rng.integers(70, 1400))
    G = int(rng.choice([0, 0, 32, 64, 96, 128, 256, 512]))
    keep = float(rng.choice([0.05, 0.1, 0.25, 0.5, 1.0]))
    say(f"random config seed={seed}: H={H} Hkv={Hkv} n={n} d={d} G={G} keep={keep}")
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    Q = torch.randn(1, H, n, d, generator=g).to(torch.bfloat16)
    K = torch.randn(1, Hkv, n, d, generator=g).to(torch.bfloat16)
    V = torch.randn(1, Hkv, n, d, generator=g).to(torch.bfloat16)
    K[:, :, 3::7] *= 2.0
    k = oracle.num_keep(n, keep)
    rep = H // Hkv
    with pc.Context(1, H, n, d, torch.bfloat16, group_size=G, kv_heads=Hkv) as ctx:
        U = ctx.groups
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        idx = ctx.select(q, k_, keep)
        O = ctx.attn(q, k_, v, idx)
        Od, idx2 = ctx.refresh_dense(q, k_, v, keep)
        torch.cuda.synchronize()
    assert idx.shape == (1, H, U, k)
    idx_host = idx.cpu().numpy()
    for h in range(H):
        qh, kh, vh = f64(Q[0, h]), f64(K[0, h // rep]), f64(V[0, h // rep])
        s64 = oracle.column_scores(qh, kh, group_size=G)
        for u in range(U):
            assert_idx_matches(idx_host[0, h, u], s64[u], k, f"seed {seed} head {h} group {u}")
            assert_idx_matches(idx2[0, h, u].cpu().numpy(), s64[u], k, f"seed {seed} refresh_dense head {h} group {u}")
        want = oracle.sparse_attention_masked(qh, kh, vh, idx_host[0, h], group_size=G)
        assert_close(O[0, h], want, "bf16", f"seed {seed} attn head {h}")
        assert_close(Od[0, h], oracle.dense_attention(qh, kh, vh), "bf16", f"seed {seed} dense head {h}")
