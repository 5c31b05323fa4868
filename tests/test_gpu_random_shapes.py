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
    # the oracle's scores and column sets come first; the attention runs through the oracle's sets
    s64 = [oracle.column_scores(f64(Q[0, h]), f64(K[0, h // rep]), group_size=G) for h in range(H)]
    oidx = np.stack([oracle.topk_columns(s64[h], k) for h in range(H)])[None]
    with pc.Context(1, H, n, d, torch.bfloat16, group_size=G, kv_heads=Hkv) as ctx:
        U = ctx.groups
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        idx = ctx.select(q, k_, keep)
        O = ctx.attn(q, k_, v, torch.from_numpy(oidx).to(torch.int32).to(DEV))
        Od, idx2 = ctx.refresh_dense(q, k_, v, keep)
        torch.cuda.synchronize()
    assert idx.shape == (1, H, U, k)
    idx_host = idx.cpu().numpy()
    for h in range(H):
        qh, kh, vh = f64(Q[0, h]), f64(K[0, h // rep]), f64(V[0, h // rep])
        for u in range(U):
            assert_idx_matches(idx_host[0, h, u], s64[h][u], k, f"seed {seed} head {h} group {u}")
            assert_idx_matches(idx2[0, h, u].cpu().numpy(), s64[h][u], k, f"seed {seed} refresh_dense head {h} group {u}")
        want = oracle.sparse_attention_masked(qh, kh, vh, oidx[0, h], group_size=G)
        assert_close(O[0, h], want, "bf16", f"seed {seed} attn head {h}")
        assert_close(Od[0, h], oracle.dense_attention(qh, kh, vh), "bf16", f"seed {seed} dense head {h}")


def _group_cases():
    rng = np.random.default_rng(2606)
    out = []
    # the small-group kernel walks over tiles of 32 columns through 3 (G = 128, 32) or 2 (G = 64)
    # LDS slots, its loop unrolled over the slots: every remainder, exact and ragged, both head dims
    for G in (128, 64, 32):
        for tiles in range(1, 9):
            for ragged in (0, int(rng.integers(1, 32))):
                k = (tiles - 1) * 32 + (ragged if ragged else 32)
                n = int(max(k, G + 1) + rng.integers(0, 200))
                d = 128 if (tiles + G // 32) % 2 else 64
                out.append((n, d, G, k))
    out += [(33, 128, 32, 1), (33, 64, 32, 33), (65, 128, 64, 2), (129, 64, 128, 129)]      # a last group of one row
    return out


@pytest.mark.parametrize("n,d,G,k", _group_cases())
def test_small_group_attention_every_tile_remainder(n, d, G, k):
    say(f"sweep group attn n={n} d={d} G={G} k={k}")
    H = 2
    g = torch.Generator(device="cpu")
    g.manual_seed(n * 17 + k + G)
    Q, K, V = (torch.randn(1, H, n, d, generator=g).to(torch.bfloat16) for _ in range(3))
    U = -(-n // G)
    idx = random_idx(n, k, H * U, seed=n + k + G).view(1, H, U, k)
    with pc.Context(1, H, n, d, torch.bfloat16, group_size=G) as ctx:
        assert ctx.groups == U
        O = ctx.attn(Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV))
        torch.cuda.synchronize()
    for h in range(H):
        q, k_, v = f64(Q[0, h]), f64(K[0, h]), f64(V[0, h])
        for u in range(U):
            lo, hi = u * G, min(n, (u + 1) * G)
            want = oracle.sparse_attention_masked(q[lo:hi], k_, v, idx[0, h, u].numpy())
            assert_close(O[0, h, lo:hi], want, "bf16", f"sweep group attn n={n} G={G} k={k} head {h} group {u}")


@pytest.mark.parametrize("n,d,G", [
    # the column pass streams 64-row Q tiles through 3 LDS slots (loop unrolled by 3) against blocks
    # of 256 keys: every remainder of the tile count, ragged last tiles, fewer rows than a tile
    (1, 128, 0), (5, 64, 0), (63, 128, 0), (64, 64, 0), (65, 128, 0), (128, 128, 0), (129, 64, 0), (191, 128, 0),
    (192, 64, 0), (193, 128, 0), (255, 128, 0), (256, 64, 0), (257, 128, 0), (300, 128, 0), (449, 64, 0), (515, 128, 0),
    (193, 128, 32), (300, 64, 64), (449, 128, 128), (515, 64, 32), (700, 128, 96)])
def test_scores_every_tile_remainder(n, d, G):
    say(f"sweep scores n={n} d={d} G={G}")
    H = 2
    g = torch.Generator(device="cpu")
    g.manual_seed(n * 29 + d + G)
    Q, K = (torch.randn(1, H, n, d, generator=g).to(torch.bfloat16) for _ in range(2))
    K[:, :, ::13] *= 2.5
    with pc.Context(1, H, n, d, torch.bfloat16, group_size=G) as ctx:
        s = ctx.scores(Q.to(DEV), K.to(DEV))
        torch.cuda.synchronize()
    for h in range(H):
        want = oracle.column_scores(f64(Q[0, h]), f64(K[0, h]), group_size=G)
        got = f64(s[0, h])
        assert got.shape == want.shape
        assert np.abs(got.sum(axis=1) - 1.0).max() < 1e-5
        assert (np.abs(got - want) / want).max() < 2e-5, f"sweep scores n={n} G={G} head {h}"
