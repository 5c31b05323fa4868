"""GPU parity for group-wise column sets (Sec. 3.3: one column set per query group G_u, the
index tensor S[i, :] shared by the rows of a group): scores, select and attention against the
fp64 oracle, with groups of whole query blocks and a ragged last group."""

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


def rand_qkv(B, H, n, d, dtype, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return tuple(torch.randn(B, H, n, d, generator=g, dtype=torch.float32).to(dtype) for _ in range(3))


def kind_of(dtype):
    return "bf16" if dtype == torch.bfloat16 else "f32"


GROUP_CASES = [
    # B, H, n, d, dtype, group_size  (bf16 groups are multiples of 256 rows, f32 of 128)
    (1, 2, 1000, 128, torch.bfloat16, 256),     # 4 groups, the last one ragged (232 rows)
    (2, 1, 1024, 128, torch.bfloat16, 512),     # 2 full groups, batch 2
    (1, 3, 800, 64, torch.bfloat16, 256),       # head_dim 64, ragged
    (1, 2, 500, 64, torch.float32, 128),        # fp32 mode: 4 groups, last ragged
    (1, 1, 384, 128, torch.float32, 256),       # fp32 mode, groups of two query blocks
    (1, 2, 1000, 128, torch.bfloat16, 128),     # the paper's group sizes: small-group kernel
    (1, 2, 600, 128, torch.bfloat16, 64),
    (1, 2, 500, 128, torch.bfloat16, 32),       # 16 groups, the last one of 20 rows
    (1, 2, 300, 64, torch.bfloat16, 32),        # head_dim 64
    (1, 1, 1000, 64, torch.bfloat16, 384),      # 3 blocks of 128 per group
    (1, 1, 980, 128, torch.bfloat16, 96),       # blocks of 32; the last tile's second half is empty
]


@pytest.mark.parametrize("B,H,n,d,dtype,G", GROUP_CASES)
def test_group_scores_match_oracle(B, H, n, d, dtype, G):
    say(f"group scores case B={B} H={H} n={n} d={d} {dtype} G={G}")
    Q, K, _ = rand_qkv(B, H, n, d, dtype, seed=5000 + n + G)
    K[:, :, ::17] *= 2.5
    U = -(-n // G)
    with pc.Context(B, H, n, d, dtype, group_size=G) as ctx:
        assert ctx.groups == U
        s1 = ctx.scores(Q.to(DEV), K.to(DEV))
        s2 = ctx.scores(Q.to(DEV), K.to(DEV))
        torch.cuda.synchronize()
    assert torch.equal(s1, s2)                      # fixed summation order
    assert s1.shape == (B, H, U, n)
    for b in range(B):
        for h in range(H):
            want = oracle.column_scores(f64(Q[b, h]), f64(K[b, h]), group_size=G)
            got = f64(s1[b, h])
            assert want.shape == got.shape
            assert np.abs(got.sum(axis=1) - 1.0).max() < 1e-5       # every group's scores sum to one
            rel = np.abs(got - want) / want
            assert rel.max() < 2e-5, f"group scores b{b} h{h}: worst relative error {rel.max():.3e}"


@pytest.mark.parametrize("B,H,n,d,dtype,G", GROUP_CASES)
def test_group_attention_matches_oracle(B, H, n, d, dtype, G):
    k = max(1, n // 7)
    say(f"group attn case B={B} H={H} n={n} d={d} {dtype} G={G} k={k}")
    Q, K, V = rand_qkv(B, H, n, d, dtype, seed=6000 + n + G)
    U = -(-n // G)
    idx = random_idx(n, k, B * H * U, seed=n * 3 + G).view(B, H, U, k)      # a different set per group
    with pc.Context(B, H, n, d, dtype, group_size=G) as ctx:
        O = ctx.attn(Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV))
        torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            want = oracle.sparse_attention_masked(f64(Q[b, h]), f64(K[b, h]), f64(V[b, h]), idx[b, h].numpy(),
                                                  group_size=G)
            assert_close(O[b, h], want, kind_of(dtype), f"group attn b{b} h{h}")


@pytest.mark.parametrize("n,d,dtype,G,keep", [
    (1000, 128, torch.bfloat16, 256, 0.1), (768, 64, torch.bfloat16, 256, 0.25), (500, 64, torch.float32, 128, 0.2),
    (700, 128, torch.bfloat16, 128, 0.15), (400, 128, torch.bfloat16, 32, 0.2)])
def test_group_select_then_attention(n, d, dtype, G, keep):
    B, H = 1, 2
    say(f"group select case n={n} d={d} {dtype} G={G} keep={keep}")
    Q, K, V = rand_qkv(B, H, n, d, dtype, seed=7000 + n)
    K[:, :, 5::13] *= 2.5
    U = -(-n // G)
    k = oracle.num_keep(n, keep)
    # the oracle's own scores and column sets first: the attention below runs through THEM, so
    # nothing the oracle consumes comes from the GPU
    s64 = [oracle.column_scores(f64(Q[0, h]), f64(K[0, h]), group_size=G) for h in range(H)]
    oidx = np.stack([oracle.topk_columns(s64[h], k) for h in range(H)])[None]
    with pc.Context(B, H, n, d, dtype, group_size=G) as ctx:
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        idx = ctx.select(q, k_, keep)
        again = ctx.select(None, None, keep, refresh=False)          # reuse step: the cached pattern
        O = ctx.attn(q, k_, v, torch.from_numpy(oidx).to(torch.int32).to(DEV))
        torch.cuda.synchronize()
    assert idx.shape == (B, H, U, k)
    assert torch.equal(idx, again)
    idx_host = idx.cpu().numpy()
    for h in range(H):
        for u in range(U):
            assert_idx_matches(idx_host[0, h, u], s64[h][u], k, f"select head {h} group {u}")
        want = oracle.sparse_attention_masked(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h]), oidx[0, h], group_size=G)
        assert_close(O[0, h], want, kind_of(dtype), f"group select+attn head {h}")


def test_groups_differ_from_one_set_per_head():
    """Planted structure: the first half of the queries is aligned with one set of keys, the
    second half with another; group-wise selection must find a different set per group."""
    B, H, n, d, G = 1, 1, 512, 128, 256
    say("group planted case")
    g = torch.Generator(device="cpu")
    g.manual_seed(99)
    Q = torch.randn(B, H, n, d, generator=g) * 0.1
    K = torch.randn(B, H, n, d, generator=g) * 0.1
    a = torch.randn(d, generator=g)
    bvec = torch.randn(d, generator=g)
    Q[0, 0, :256] += a
    Q[0, 0, 256:] += bvec
    cols_a = torch.arange(3, 200, 7)
    cols_b = torch.arange(300, 500, 7)
    K[0, 0, cols_a] += a
    K[0, 0, cols_b] += bvec
    Q, K = Q.to(torch.bfloat16), K.to(torch.bfloat16)
    k = cols_a.numel()
    with pc.Context(B, H, n, d, torch.bfloat16, group_size=G) as ctx:
        scores = ctx.scores(Q.to(DEV), K.to(DEV))
        idx = ctx.topk(scores, k)
        torch.cuda.synchronize()
    assert set(idx[0, 0, 0].tolist()) == set(cols_a.tolist())
    assert set(idx[0, 0, 1].tolist()) == set(cols_b.tolist())


def test_layer_stack_follows_the_schedule():
    """Three layers, eight steps, refresh at steps 0 and 3: every layer's output at every step
    equals what the single calls give, and the pattern only changes at refresh steps."""
    from paper_2605_20813_amd import schedule as sch
    B, H, n, d, keep, L, T = 1, 2, 512, 128, 0.2, 3, 8
    say("layer stack case")
    steps = sch.refresh_steps(T, 0.5, 2)
    assert steps == [0, 3]
    g = torch.Generator(device="cpu")
    g.manual_seed(123)
    base = [tuple(torch.randn(B, H, n, d, generator=g).to(torch.bfloat16).to(DEV) for _ in range(3)) for _ in range(L)]
    out = [torch.empty(B, H, n, d, dtype=torch.bfloat16, device=DEV) for _ in range(L)]
    with sch.LayerStack(L, B, H, n, d, torch.bfloat16, keep, steps) as stack, \
            pc.Context(B, H, n, d, torch.bfloat16) as ref:
        patterns = [None] * L
        for t in range(T):
            # the activations drift a little from step to step
            qkv = [tuple((x.float() * (1.0 + 0.01 * t)).to(torch.bfloat16) for x in base[l]) for l in range(L)]
            assert stack.step(t, qkv, out) == (L if t in steps else 0)
            for l in range(L):
                Q, K, V = qkv[l]
                if t in steps:
                    patterns[l] = ref.select(Q, K, keep).clone()
                assert torch.equal(stack.idx[l], patterns[l])
                assert torch.equal(out[l], ref.attn(Q, K, V, patterns[l]))
        torch.cuda.synchronize()
    # dense output at refresh steps
    with sch.LayerStack(1, B, H, n, d, torch.bfloat16, keep, [0], dense_at_refresh=True) as stack, \
            pc.Context(B, H, n, d, torch.bfloat16) as ref:
        Q, K, V = base[0]
        stack.step(0, [base[0]], out[:1])
        assert torch.equal(out[0], ref.attn_dense(Q, K, V))
        stack.step(1, [base[0]], out[:1])
        assert torch.equal(out[0], ref.attn(Q, K, V, stack.idx[0]))
        torch.cuda.synchronize()
