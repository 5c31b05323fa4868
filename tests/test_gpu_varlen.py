"""Variable-length batches (pulsecol_set_seq_lens): every batch element against the oracle run on
that element alone, at its own length.  The padding of the inputs holds NaN, the outputs are
pre-filled with NaN: whatever is read from or written to the padding shows."""

import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2605_20813_amd import pulsecol as pc
from paper_2605_20813_amd import workloads as wl
from parity_util import assert_close, assert_idx_matches, f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def kind_of(dtype):
    return "bf16" if dtype == torch.bfloat16 else "f32"


def padded_qkv(B, H, n, d, dtype, lens, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    Q, K, V = (torch.randn(B, H, n, d, generator=g, dtype=torch.float32) for _ in range(3))
    K[:, :, 3::11] *= 2.5
    Q, K, V = (t.to(dtype) for t in (Q, K, V))
    for b, L in enumerate(lens):
        for t in (Q, K, V):
            t[b, :, L:] = float("nan")
    return Q, K, V


CASES = [
    # B, H, n, d, dtype, G, lens, keep
    (3, 2, 700, 128, torch.bfloat16, 0, (700, 333, 64), 0.2),          # main kernel, one set per head
    (3, 2, 700, 128, torch.bfloat16, 256, (700, 300, 257), 0.2),       # main kernel, group-wise
    (3, 2, 640, 128, torch.bfloat16, 64, (640, 130, 63), 0.1),         # small-group kernel
    (2, 3, 520, 64, torch.bfloat16, 32, (519, 33), 0.25),              # head_dim 64, one-wave groups
    (2, 2, 384, 64, torch.float32, 0, (384, 130), 0.25),               # fp32 kernels
    (2, 2, 384, 128, torch.float32, 128, (200, 384), 0.2),
    (1, 2, 300, 128, torch.bfloat16, 0, (1,), 0.5),                    # a single real position
]


@pytest.mark.parametrize("B,H,n,d,dtype,G,lens,keep", CASES)
def test_every_batch_element_matches_the_oracle_at_its_own_length(B, H, n, d, dtype, G, lens, keep):
    say(f"varlen case B={B} H={H} n={n} d={d} {dtype} G={G} lens={lens} keep={keep}")
    Q, K, V = padded_qkv(B, H, n, d, dtype, lens, seed=n + d + G)
    kind = kind_of(dtype)
    k = oracle.num_keep(n, keep)
    # the oracle first, per element on its own rows: scores, column sets, and the sets the attention will be fed
    s64, oidx = {}, {}
    for b, L in enumerate(lens):
        for h in range(H):
            s64[b, h] = oracle.column_scores(f64(Q[b, h, :L]), f64(K[b, h, :L]), group_size=G)
            oidx[b, h] = oracle.topk_columns(s64[b, h], oracle.num_keep(L, keep))
    with pc.Context(B, H, n, d, dtype, group_size=G) as ctx:
        U = ctx.groups
        ctx.set_seq_lens(lens)
        idx_in = torch.full((B, H, U, k), -1, dtype=torch.int32)
        for (b, h), cols in oidx.items():
            idx_in[b, h, :cols.shape[0], :cols.shape[1]] = torch.from_numpy(cols).to(torch.int32)
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        sc = torch.full((B, H, U, n), float("nan"), dtype=torch.float32, device=DEV)
        ctx.scores(q, k_, scores_out=sc)
        idx = torch.full((B, H, U, k), -7, dtype=torch.int32, device=DEV)
        ctx.select(q, k_, keep, idx_out=idx)
        again = ctx.select(None, None, keep, refresh=False)
        nan_like = lambda: torch.full((B, H, n, d), float("nan"), dtype=dtype, device=DEV)
        O = ctx.attn(q, k_, v, idx_in.to(DEV), O=nan_like())
        lse = torch.full((B, H, n), float("nan"), dtype=torch.float32, device=DEV)
        Od = ctx.attn_dense(q, k_, v, O=nan_like(), lse_out=lse)
        Or, idx_r = ctx.refresh_dense(q, k_, v, keep, O=nan_like())
        torch.cuda.synchronize()
    assert torch.equal(idx, again)
    idx_h, idx_rh = idx.cpu().numpy(), idx_r.cpu().numpy()
    for b, L in enumerate(lens):
        kb = oracle.num_keep(L, keep)
        Ub = -(-L // G) if G else 1
        for h in range(H):
            got = f64(sc[b, h, :Ub, :L])
            assert np.isfinite(got).all()
            rel = np.abs(got - s64[b, h]) / s64[b, h]
            assert rel.max() < 2e-5, f"scores b{b} h{h}: {rel.max():.3e}"
            for u in range(Ub):
                assert_idx_matches(idx_h[b, h, u, :kb], s64[b, h][u], kb, f"select b{b} h{h} u{u}")
                assert_idx_matches(idx_rh[b, h, u, :kb], s64[b, h][u], kb, f"refresh_dense b{b} h{h} u{u}")
            assert (idx_h[b, h, :Ub, kb:] == -1).all() and (idx_h[b, h, Ub:] == -1).all()
            assert (idx_rh[b, h, :Ub, kb:] == -1).all() and (idx_rh[b, h, Ub:] == -1).all()
            qh, kh, vh = f64(Q[b, h, :L]), f64(K[b, h, :L]), f64(V[b, h, :L])
            assert_close(O[b, h, :L], oracle.sparse_attention_masked(qh, kh, vh, oidx[b, h], group_size=G), kind, f"attn b{b} h{h}")
            want_d = oracle.dense_attention(qh, kh, vh)
            assert_close(Od[b, h, :L], want_d, kind, f"dense b{b} h{h}")
            assert_close(Or[b, h, :L], want_d, kind, f"refresh_dense output b{b} h{h}")
            z = oracle.attention_logits(qh, kh)
            want_lse = np.log(np.exp(z - z.max(1, keepdims=True)).sum(1)) + z.max(1)
            assert np.abs(f64(lse[b, h, :L]) - want_lse).max() < 2e-5 * max(1.0, np.abs(want_lse).max())
            # the padding rows of the outputs were never written
            for out in (O, Od, Or):
                assert torch.isnan(out[b, h, L:].float()).all()
            assert torch.isnan(lse[b, h, L:]).all()


@pytest.mark.parametrize("n,k,lens", [
    (1000, 300, (1000, 431, 10)),          # the row held in registers (n a multiple of 4), lengths that are not
    (1003, 300, (1003, 502, 299)),         # the streaming kernel (n not a multiple of 4)
    (4096, 512, (4096, 4095, 2049)),       # several register groups per lane
])
def test_topk_on_given_scores_and_ties_per_element(n, k, lens):
    B, H = 3, 2
    say(f"varlen top-k case n={n} k={k} lens={lens}")
    scores = wl.random_scores(B * H, n, seed=99, ties=True).view(B, H, 1, n)
    for b, L in enumerate(lens):
        scores[b, :, :, L:] = float("nan")            # what lies behind an element's end must not matter
    with pc.Context(B, H, n, 128, torch.bfloat16) as ctx:
        ctx.set_seq_lens(lens)
        idx = ctx.topk(scores.to(DEV), k).cpu().numpy()
        ctx.set_seq_lens(None)
        plain = ctx.topk(torch.nan_to_num(scores, nan=0.0).to(DEV), k).cpu().numpy()
    for b, L in enumerate(lens):
        kb = min(k, L)
        for h in range(H):
            want = oracle.topk_columns(f64(scores[b, h, 0, :L])[None], kb)[0]
            assert np.array_equal(idx[b, h, 0, :kb], want), (b, h)
            assert (idx[b, h, 0, kb:] == -1).all()
    # back at fixed length every row selects k of all n scores again
    for h in range(H):
        want = oracle.topk_columns(f64(torch.nan_to_num(scores, nan=0.0)[0, h, 0])[None], k)[0]
        assert np.array_equal(plain[0, h, 0], want)


def test_lengths_are_checked_and_drop_the_cached_pattern():
    B, H, n, d = 2, 2, 256, 128
    say("varlen error paths")
    Q, K, V = padded_qkv(B, H, n, d, torch.bfloat16, (256, 256), seed=5)
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx:
        for bad in ((0, 10), (257, 10), (-3, 5)):
            with pytest.raises(pc.PulseColError) as e:
                ctx.set_seq_lens(bad)
            assert e.value.status == pc.ERR_INVALID_ARG
        with pytest.raises(ValueError):
            ctx.set_seq_lens((10,))
        full = ctx.select(Q.to(DEV), K.to(DEV), 0.25).clone()
        ctx.set_seq_lens((256, 100))
        with pytest.raises(pc.PulseColError) as e:
            ctx.select(None, None, 0.25, refresh=False)
        assert e.value.status == pc.ERR_NO_PATTERN
        part = ctx.select(Q.to(DEV), K.to(DEV), 0.25).clone()
        torch.cuda.synchronize()
        assert torch.equal(part[0], full[0])                       # an element at full length: as without lengths
        assert (part[1, :, :, 25:] == -1).all() and (part[1, :, :, :25] >= 0).all() and (part[1, :, :, :25] < 100).all()


@pytest.mark.timeout(600)
def test_batch_of_four_at_workload_scale():
    """B = 4 at the 16K workload's shape (8 heads), elements of 16384 / 12000 / 8229 / 1000 positions:
    sampled query rows of every element against the oracle at the element's own length."""
    w = wl.WORKLOADS["llada_16k"]
    B, H, n, d, keep = 4, 8, w.seq, w.head_dim, 0.10
    lens = (16384, 12000, 8229, 1000)
    say("varlen workload-scale case: generating")
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed)
    Q, K, V = (torch.randn(B, H, n, d, generator=g).to(torch.bfloat16) for _ in range(3))
    K[:, :, ::19] *= 2.5
    k = oracle.num_keep(n, keep)
    rng = np.random.default_rng(1)
    idx_in = torch.full((B, H, 1, k), -1, dtype=torch.int32)
    for b, L in enumerate(lens):
        kb = oracle.num_keep(L, keep)
        for h in range(H):
            idx_in[b, h, 0, :kb] = torch.from_numpy(np.sort(rng.choice(L, size=kb, replace=False)).astype(np.int32))
    with pc.Context(B, H, n, d, torch.bfloat16, max_keep_ratio=keep) as ctx:
        ctx.set_seq_lens(lens)
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        idx = ctx.select(q, k_, keep)
        O = ctx.attn(q, k_, v, idx_in.to(DEV))
        Od = ctx.attn_dense(q, k_, v)
        torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    for b, L in enumerate(lens):
        kb = oracle.num_keep(L, keep)
        h = (3 * b + 1) % H
        rows = np.unique(np.concatenate([[0, L - 1, min(255, L - 1), min(256, L - 1)], rng.integers(0, L, 24)]))
        say(f"  element {b} (length {L}): oracle rows of head {h}")
        qh, kh, vh = f64(Q[b, h, :L]), f64(K[b, h, :L]), f64(V[b, h, :L])
        assert_close(O[b, h][rows], oracle.sparse_attention_masked(qh, kh, vh, idx_in[b, h, :, :kb].numpy(), rows=rows), "bf16", f"attn b{b}")
        assert_close(Od[b, h][rows], oracle.dense_attention(qh, kh, vh, rows=rows), "bf16", f"dense b{b}")
        row = idx_h[b, :, 0, :kb]
        assert (row[:, 1:] > row[:, :-1]).all() and row.min() >= 0 and row.max() < L
        assert (idx_h[b, :, 0, kb:] == -1).all()
        if L <= 8229:       # the whole selection of one head, where the oracle's scores are affordable
            s64 = oracle.column_scores(qh, kh)[0]
            assert_idx_matches(idx_h[b, h, 0, :kb], s64, kb, f"select b{b} h{h}")
