"""Block-sparse attention and block selection (the block-mask formulation of Sec. 3.1 that the
paper contrasts column sparsity with) against the fp64 oracle."""

import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2605_20813_amd import pulsecol as pc
from parity_util import assert_close, assert_idx_matches, f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
KEY_BLOCK = 64


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def rand_qkv(B, H, n, d, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    Q, K, V = (torch.randn(B, H, n, d, generator=g, dtype=torch.float32) for _ in range(3))
    K[:, :, 128:192] *= 2.0                       # one heavy key block
    return tuple(t.to(torch.bfloat16) for t in (Q, K, V))


def random_blocks(B, H, U, nblocks, kb, seed, sort=True):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    out = torch.empty(B, H, U, kb, dtype=torch.int32)
    for b in range(B):
        for h in range(H):
            for u in range(U):
                sel = torch.randperm(nblocks, generator=g)[:kb]
                out[b, h, u] = (torch.sort(sel).values if sort else sel).to(torch.int32)
    return out


@pytest.mark.parametrize("B,H,n,d,G,kb,sort", [
    (1, 3, 1024, 128, 0, 5, True),
    (2, 2, 768, 64, 256, 3, True),          # one block mask per 256-row query block, head_dim 64
    (1, 2, 1000 - 1000 % 64, 128, 512, 4, False),     # two query blocks per mask (last one ragged), blocks in any order
    (1, 2, 640, 128, 0, 10, True),          # every key block: dense attention
    (1, 9, 320, 128, 0, 1, True),           # one key block, more heads than XCDs
])
def test_block_sparse_attention_matches_oracle(B, H, n, d, G, kb, sort):
    say(f"block attn case B={B} H={H} n={n} d={d} G={G} kb={kb}")
    Q, K, V = rand_qkv(B, H, n, d, seed=n + kb)
    with pc.Context(B, H, n, d, torch.bfloat16, group_size=G) as ctx:
        U = ctx.groups
        blocks = random_blocks(B, H, U, n // KEY_BLOCK, kb, seed=n * 3 + kb, sort=sort)
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        O = ctx.attn_block(q, k_, v, blocks.to(DEV))
        # the same columns through the column-sparse call of the same (hand-scheduled) kernel
        ctx.set_attn_block(256)
        cols = torch.from_numpy(np.stack([[oracle.block_columns(blocks[b, h].numpy(), KEY_BLOCK) for h in range(H)]
                                          for b in range(B)])).to(torch.int32)
        Oc = ctx.attn(q, k_, v, cols.to(DEV))
        torch.cuda.synchronize()
    assert torch.equal(O, Oc)               # same keys in the same tile positions: bit-identical
    for b in range(B):
        for h in range(H):
            want = oracle.block_sparse_attention(f64(Q[b, h]), f64(K[b, h]), f64(V[b, h]), blocks[b, h].numpy(), KEY_BLOCK,
                                                 group_size=G)
            assert_close(O[b, h], want, "bf16", f"block attn b{b} h{h}")
    if kb == n // KEY_BLOCK and G == 0:
        for h in range(H):
            assert_close(O[0, h], oracle.dense_attention(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h])), "bf16", "all blocks")


@pytest.mark.parametrize("n,d,G,keep", [(1024, 128, 0, 0.2), (1536, 64, 256, 0.1), (2048, 128, 512, 0.26)])
def test_block_selection_matches_oracle(n, d, G, keep):
    B, H = 1, 3
    say(f"block select case n={n} d={d} G={G} keep={keep}")
    Q, K, V = rand_qkv(B, H, n, d, seed=n + 7)
    kb = oracle.num_keep(n // KEY_BLOCK, keep)
    assert pc.num_keep_blocks(n, keep) == kb
    # the oracle's block masses and sets first; the attention then runs through the oracle's sets
    mass = [oracle.block_scores(f64(Q[0, h]), f64(K[0, h]), KEY_BLOCK, group_size=G) for h in range(H)]
    oblk = np.stack([oracle.topk_columns(mass[h], kb) for h in range(H)])[None]
    with pc.Context(B, H, n, d, torch.bfloat16, group_size=G) as ctx:
        U = ctx.groups
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        got = ctx.select_blocks(q, k_, keep)
        again = ctx.select_blocks(q, k_, keep)
        O = ctx.attn_block(q, k_, v, torch.from_numpy(oblk).to(torch.int32).to(DEV))
        torch.cuda.synchronize()
    assert got.shape == (B, H, U, kb) and torch.equal(got, again)
    for h in range(H):
        for u in range(U):
            assert_idx_matches(got[0, h, u].cpu().numpy(), mass[h][u], kb, f"block select h{h} u{u}")
        want = oracle.block_sparse_attention(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h]), oblk[0, h], KEY_BLOCK, group_size=G)
        assert_close(O[0, h], want, "bf16", f"block select+attn h{h}")
    assert 2 in got[0, :, 0].cpu().numpy()          # the planted heavy key block (keys 128..191)


def test_block_mode_limits():
    say("block mode limits")
    Q, K, V = (t.to(DEV) for t in rand_qkv(1, 2, 512, 128, seed=3))
    blocks = random_blocks(1, 2, 1, 8, 2, seed=4).to(DEV)
    with pc.Context(1, 2, 512, 128, torch.bfloat16) as ctx:
        L = pc.lib()
        for kb in (0, 9):
            st = L.pulsecol_attn_block(ctx._h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), blocks.data_ptr(), kb, Q.data_ptr(), None)
            assert st == pc.ERR_INVALID_ARG
        ctx.set_validation(True)
        bad = blocks.clone()
        bad[0, 1, 0, 1] = 8
        with pytest.raises(pc.PulseColError) as e:
            ctx.attn_block(Q, K, V, bad)
        assert e.value.status == pc.ERR_BAD_INDEX
        ctx.set_validation(False)
        ctx.set_seq_lens((300,))
        with pytest.raises(pc.PulseColError) as e:
            ctx.attn_block(Q, K, V, blocks)
        assert e.value.status == pc.ERR_UNSUPPORTED
    for kw in (dict(seq=500), dict(group_size=64), dict(dtype=torch.float32, group_size=128)):
        args = dict(batch=1, heads=2, seq=512, head_dim=128, dtype=torch.bfloat16, group_size=0)
        args.update(kw)
        with pc.Context(args["batch"], args["heads"], args["seq"], args["head_dim"], args["dtype"], group_size=args["group_size"]) as ctx:
            n = args["seq"]
            t = torch.zeros(1, 2, n, 128, dtype=args["dtype"], device=DEV)
            st = pc.lib().pulsecol_attn_block(ctx._h, t.data_ptr(), t.data_ptr(), t.data_ptr(), blocks.data_ptr(), 1, t.data_ptr(), None)
            assert st == pc.ERR_UNSUPPORTED, kw
    assert pc.num_keep_blocks(500, 0.1) == -1 and pc.num_keep_blocks(4096, 0.1) == 6 and pc.num_keep_blocks(64, 0.01) == 1
