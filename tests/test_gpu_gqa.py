"""GPU parity for the grouped-query layout (fewer K/V heads than query heads, as in the
Dream-style models the paper also evaluates): query head h reads K/V head h // (H / H_kv);
patterns stay per query head.  The oracle needs no change: it is called per query head with
the K/V head that head reads."""

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


def rand(shape, dtype, g):
    return torch.randn(*shape, generator=g, dtype=torch.float32).to(dtype)


def kind_of(dtype):
    return "bf16" if dtype == torch.bfloat16 else "f32"


CASES = [
    # B, H, Hkv, n, d, dtype, group_size
    (1, 8, 2, 700, 128, torch.bfloat16, 0),
    (2, 4, 1, 520, 64, torch.bfloat16, 0),       # multi-query: one K/V head
    (1, 6, 3, 600, 128, torch.bfloat16, 128),    # with query groups: small-group kernel
    (1, 4, 2, 1000, 128, torch.bfloat16, 256),
    (1, 4, 2, 300, 64, torch.float32, 0),
]


@pytest.mark.parametrize("B,H,Hkv,n,d,dtype,G", CASES)
def test_gqa_select_attention_and_dense(B, H, Hkv, n, d, dtype, G):
    say(f"gqa case B={B} H={H} Hkv={Hkv} n={n} d={d} {dtype} G={G}")
    g = torch.Generator(device="cpu")
    g.manual_seed(9000 + n + H)
    Q = rand((B, H, n, d), dtype, g)
    K = rand((B, Hkv, n, d), dtype, g)
    V = rand((B, Hkv, n, d), dtype, g)
    K[:, :, 7::19] *= 2.5
    keep = 0.15
    k = oracle.num_keep(n, keep)
    rep = H // Hkv
    with pc.Context(B, H, n, d, dtype, group_size=G, kv_heads=Hkv) as ctx:
        U = ctx.groups
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        sc = ctx.scores(q, k_)
        idx = ctx.select(q, k_, keep)
        given = random_idx(n, k, B * H * U, seed=n + 5).view(B, H, U, k)
        O = ctx.attn(q, k_, v, given.to(DEV))
        Od = ctx.attn_dense(q, k_, v)
        torch.cuda.synchronize()
    assert sc.shape == (B, H, U, n) and idx.shape == (B, H, U, k)
    idx_host = idx.cpu().numpy()
    for b in range(B):
        for h in range(H):
            qh, kh, vh = f64(Q[b, h]), f64(K[b, h // rep]), f64(V[b, h // rep])
            s64 = oracle.column_scores(qh, kh, group_size=G)
            rel = np.abs(f64(sc[b, h]) - s64) / s64
            assert rel.max() < 2e-5, f"gqa scores b{b} h{h}: {rel.max():.3e}"
            for u in range(U):
                assert_idx_matches(idx_host[b, h, u], s64[u], k, f"gqa select b{b} h{h} u{u}")
            want = oracle.sparse_attention_masked(qh, kh, vh, given[b, h].numpy(), group_size=G)
            assert_close(O[b, h], want, kind_of(dtype), f"gqa attn b{b} h{h}")
            assert_close(Od[b, h], oracle.dense_attention(qh, kh, vh), kind_of(dtype), f"gqa dense b{b} h{h}")


def test_gqa_equals_expanded_multi_head():
    """The same numbers as multi-head attention on K/V with every head repeated."""
    B, H, Hkv, n, d = 1, 8, 2, 640, 128
    say("gqa expanded case")
    g = torch.Generator(device="cpu")
    g.manual_seed(77)
    Q = rand((B, H, n, d), torch.bfloat16, g).to(DEV)
    K = rand((B, Hkv, n, d), torch.bfloat16, g).to(DEV)
    V = rand((B, Hkv, n, d), torch.bfloat16, g).to(DEV)
    Kx = K.repeat_interleave(H // Hkv, dim=1).contiguous()
    Vx = V.repeat_interleave(H // Hkv, dim=1).contiguous()
    with pc.Context(B, H, n, d, torch.bfloat16, kv_heads=Hkv) as a, pc.Context(B, H, n, d, torch.bfloat16) as m:
        ia, im = a.select(Q, K, 0.1), m.select(Q, Kx, 0.1)
        assert torch.equal(ia, im)
        assert torch.equal(a.attn(Q, K, V, ia), m.attn(Q, Kx, Vx, im))
        assert torch.equal(a.attn_dense(Q, K, V), m.attn_dense(Q, Kx, Vx))
        torch.cuda.synchronize()
