"""GPU parity: every entry point of the C-ABI library against the fp64 CPU oracle, element by
element, on seeded synthetic inputs -- small and medium sizes that span several tiles and
ragged tails, plus the edge cases of the method.  Full-size cases live in
test_gpu_fullsize.py."""

import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2605_20813_amd import pulsecol as pc
from paper_2605_20813_amd import workloads as wl
from parity_util import TOL, assert_close, assert_idx_matches, f64, random_idx

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


# ---------------------------------------------------------------------------------------
# column-sparse attention
# ---------------------------------------------------------------------------------------
ATTN_CASES = [
    # B, H, n, d, dtype, k
    (1, 2, 256, 64, torch.float32, 64),        # the tiny workload's shape
    (1, 3, 1000, 128, torch.bfloat16, 137),    # ragged rows, ragged last tile
    (2, 2, 777, 128, torch.bfloat16, 64),      # exactly one tile, batch 2
    (1, 2, 777, 128, torch.bfloat16, 65),      # one column in the last tile
    (1, 1, 300, 128, torch.bfloat16, 1),       # one kept column
    (1, 2, 520, 128, torch.bfloat16, 520),     # keep everything
    (1, 9, 260, 128, torch.bfloat16, 100),     # more heads than XCDs, not a multiple of 8
    (1, 2, 600, 64, torch.bfloat16, 200),      # head_dim 64
    (1, 2, 333, 128, torch.float32, 77),       # fp32 mode, head_dim 128, ragged
    (1, 1, 130, 64, torch.float32, 33),
]


@pytest.mark.parametrize("B,H,n,d,dtype,k", ATTN_CASES)
def test_sparse_attention_matches_oracle(B, H, n, d, dtype, k):
    say(f"attn case B={B} H={H} n={n} d={d} {dtype} k={k}")
    Q, K, V = rand_qkv(B, H, n, d, dtype, seed=1000 + n + k)
    idx = random_idx(n, k, B * H, seed=n * 7 + k).view(B, H, 1, k)
    with pc.Context(B, H, n, d, dtype) as ctx:
        O = ctx.attn(Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV))
        torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            want = oracle.sparse_attention_masked(f64(Q[b, h]), f64(K[b, h]), f64(V[b, h]), idx[b, h].numpy())
            assert_close(O[b, h], want, kind_of(dtype), f"attn b{b} h{h}")


@pytest.mark.parametrize("B,H,n,d,dtype", [
    (1, 2, 256, 64, torch.float32), (1, 3, 1000, 128, torch.bfloat16), (2, 1, 257, 128, torch.bfloat16),
    (1, 2, 500, 64, torch.bfloat16), (1, 2, 333, 128, torch.float32)])
def test_dense_attention_and_lse_match_oracle(B, H, n, d, dtype):
    say(f"dense case B={B} H={H} n={n} d={d} {dtype}")
    Q, K, V = rand_qkv(B, H, n, d, dtype, seed=2000 + n)
    with pc.Context(B, H, n, d, dtype) as ctx:
        lse = torch.empty(B, H, n, dtype=torch.float32, device=DEV)
        O = ctx.attn_dense(Q.to(DEV), K.to(DEV), V.to(DEV), lse_out=lse)
        torch.cuda.synchronize()
    for b in range(B):
        for h in range(H):
            q, k_, v = f64(Q[b, h]), f64(K[b, h]), f64(V[b, h])
            assert_close(O[b, h], oracle.dense_attention(q, k_, v), kind_of(dtype), f"dense b{b} h{h}")
            Z = oracle.attention_logits(q, k_)
            m = Z.max(axis=1)
            want_lse = m + np.log(np.exp(Z - m[:, None]).sum(axis=1))
            np.testing.assert_allclose(f64(lse[b, h]), want_lse, rtol=0, atol=2e-5 * max(1.0, np.abs(want_lse).max()))


def test_keep_everything_equals_dense_on_gpu_and_oracle(attn_kernel):
    B, H, n, d = 1, 2, 640, 128
    say("keep=1 case")
    Q, K, V = rand_qkv(B, H, n, d, torch.bfloat16, seed=31)
    every = torch.arange(n, dtype=torch.int32).repeat(B, H, 1, 1)
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx:
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        Os = ctx.attn(q, k_, v, every.to(DEV))
        Od = ctx.attn_dense(q, k_, v)
        torch.cuda.synchronize()
    if attn_kernel == 256:
        assert torch.equal(Os, Od)      # the dense kernel is the scheduled one: same tiles in the same order, bit-identical
    else:
        assert (Os.float() - Od.float()).abs().max().item() <= TOL["bf16"]["max_abs"]
    for h in range(H):
        assert_close(Os[0, h], oracle.dense_attention(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h])), "bf16", "keep=1")


def test_column_order_and_repeats():
    B, H, n, d, k = 1, 2, 512, 128, 150
    say("column-order case")
    Q, K, V = rand_qkv(B, H, n, d, torch.bfloat16, seed=41)
    idx = random_idx(n, k, B * H, seed=42).view(B, H, 1, k)
    shuffled = random_idx(n, k, B * H, seed=42, sort=False).view(B, H, 1, k)
    assert torch.equal(torch.sort(shuffled, dim=-1).values, idx)
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx:
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        O1 = ctx.attn(q, k_, v, idx.to(DEV))
        O2 = ctx.attn(q, k_, v, shuffled.to(DEV))
        O1b = ctx.attn(q, k_, v, idx.to(DEV))
        # a repeated column counts twice (appendix listing semantics)
        rep = torch.tensor([5, 5, 9], dtype=torch.int32).repeat(B, H, 1, 1)
        O3 = ctx.attn(q, k_, v, rep.to(DEV))
        torch.cuda.synchronize()
    assert torch.equal(O1, O1b)                                        # run-to-run determinism
    assert (O1.float() - O2.float()).abs().max().item() <= TOL["bf16"]["max_abs"]
    for h in range(H):
        want = oracle.sparse_attention_masked(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h]), idx[0, h].numpy())
        assert_close(O2[0, h], want, "bf16", "shuffled idx")
        want3 = oracle.sparse_attention_gathered(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h]), [[5, 5, 9]])
        assert_close(O3[0, h], want3, "bf16", "repeated idx")


def test_ones_value_gives_ones_and_single_column_copies_value():
    B, H, n, d = 1, 2, 384, 128
    say("V==1 / k==1 case")
    Q, K, V = rand_qkv(B, H, n, d, torch.bfloat16, seed=51)
    idx = random_idx(n, 99, B * H, seed=52).view(B, H, 1, 99)
    one = torch.tensor([123], dtype=torch.int32).repeat(B, H, 1, 1)
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx:
        O = ctx.attn(Q.to(DEV), K.to(DEV), torch.ones_like(V).to(DEV), idx.to(DEV))
        O1 = ctx.attn(Q.to(DEV), K.to(DEV), V.to(DEV), one.to(DEV))
        torch.cuda.synchronize()
    assert (O.float() - 1.0).abs().max().item() <= 1e-2
    assert torch.equal(O1.cpu(), V[:, :, 123:124, :].expand(B, H, n, d))   # weight exactly 1.0


def test_strided_layout():
    """Tensors stored [B, n, H, d] (the projection's natural output) viewed as [B, H, n, d]."""
    B, H, n, d, k = 1, 4, 300, 128, 70
    say("strided case")
    Q, K, V = rand_qkv(B, H, n, d, torch.bfloat16, seed=61)
    idx = random_idx(n, k, B * H, seed=62).view(B, H, 1, k)

    def strided(t):
        return t.to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)

    q, k_, v = strided(Q), strided(K), strided(V)
    strides = (n * H * d, d, H * d)
    with pc.Context(B, H, n, d, torch.bfloat16, strides=strides) as ctx:
        O = torch.empty(B, n, H, d, dtype=torch.bfloat16, device=DEV).permute(0, 2, 1, 3)
        ctx.attn(q, k_, v, idx.to(DEV), O=O)
        sc = ctx.scores(q, k_)
        torch.cuda.synchronize()
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx2:
        O_packed = ctx2.attn(Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV))
        sc_packed = ctx2.scores(Q.to(DEV), K.to(DEV))
        torch.cuda.synchronize()
    assert torch.equal(O.contiguous(), O_packed)
    assert torch.equal(sc, sc_packed)


def test_padded_row_stride_with_library_allocated_output():
    """Row stride 136 (> head_dim): the output the binding allocates itself must have the
    context's strides and an allocation that holds every element the kernels store."""
    B, H, n, d, k, sn = 2, 3, 300, 128, 70, 136
    say("padded-stride case")
    Q, K, V = rand_qkv(B, H, n, d, torch.bfloat16, seed=71)
    idx = random_idx(n, k, B * H, seed=72).view(B, H, 1, k)

    def padded(t):
        buf = torch.zeros(B, H, n, sn, dtype=torch.bfloat16, device=DEV)
        buf[..., :d] = t.to(DEV)
        return buf[..., :d]

    q, k_, v = padded(Q), padded(K), padded(V)
    with pc.Context(B, H, n, d, torch.bfloat16, strides=(0, 0, sn)) as ctx:
        outs = [ctx.attn(q, k_, v, idx.to(DEV)), ctx.attn_dense(q, k_, v), ctx.refresh_dense(q, k_, v, 0.25)[0]]
        torch.cuda.synchronize()
    last_element = (B - 1) * H * n * sn + (H - 1) * n * sn + (n - 1) * sn + d       # one past the last stored element
    for O in outs:
        assert tuple(O.stride()) == (H * n * sn, n * sn, sn, 1)
        assert O.untyped_storage().nbytes() >= (O.storage_offset() + last_element) * O.element_size()
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx2:
        want = [ctx2.attn(Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV)), ctx2.attn_dense(Q.to(DEV), K.to(DEV), V.to(DEV))]
        torch.cuda.synchronize()
    assert torch.equal(outs[0].contiguous(), want[0])
    assert torch.equal(outs[1].contiguous(), want[1])
    assert torch.equal(outs[2].contiguous(), want[1])


# ---------------------------------------------------------------------------------------
# identification pass: scores, top-k, select
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("B,H,n,d,dtype", [
    (1, 2, 256, 64, torch.float32), (1, 3, 1000, 128, torch.bfloat16), (2, 2, 515, 128, torch.bfloat16),
    (1, 2, 700, 64, torch.bfloat16), (1, 2, 333, 128, torch.float32)])
def test_scores_match_oracle(B, H, n, d, dtype):
    say(f"scores case B={B} H={H} n={n} d={d} {dtype}")
    Q, K, _ = rand_qkv(B, H, n, d, dtype, seed=3000 + n)
    K[:, :, ::17] *= 2.5
    with pc.Context(B, H, n, d, dtype) as ctx:
        s1 = ctx.scores(Q.to(DEV), K.to(DEV))
        s2 = ctx.scores(Q.to(DEV), K.to(DEV))
        torch.cuda.synchronize()
    assert torch.equal(s1, s2)                                          # fixed summation order
    assert s1.shape == (B, H, 1, n)
    for b in range(B):
        for h in range(H):
            want = oracle.column_scores(f64(Q[b, h]), f64(K[b, h]))[0]
            got = f64(s1[b, h, 0])
            assert abs(got.sum() - 1.0) < 1e-5
            rel = np.abs(got - want) / want
            assert rel.max() < 2e-5, f"scores b{b} h{h}: worst relative error {rel.max():.3e}"


@pytest.mark.parametrize("rows,n,k,ties", [
    (2, 256, 64, False), (3, 1000, 137, False), (4, 5000, 1, False), (2, 5000, 5000, False),
    (3, 4096, 409, True), (2, 1023, 500, True), (1, 65536, 6553, False), (1, 65536, 6553, True),
    (2, 70001, 7000, True),
    # rows held in registers (n % 4 == 0, n <= 65536): ragged segments, every register count, k = n
    (2, 12, 12, True), (3, 16, 3, False), (2, 4100, 300, True), (3, 8192, 8192, False), (2, 16388, 1, True),
    (2, 32768, 3276, True), (2, 65532, 1000, True), (40, 65536, 6553, True),
    # more rows than resident workgroups: every workgroup walks over several rows, fetching the next
    # one while it writes the running one out (1 and 16 register groups per lane, ragged rows)
    (1300, 1020, 100, True), (700, 8200, 999, True), (300, 65536, 6553, True), (530, 40000, 4000, False)])
def test_topk_is_bit_exact_on_identical_scores(rows, n, k, ties):
    say(f"topk case rows={rows} n={n} k={k} ties={ties}")
    s = wl.random_scores(rows, n, seed=n + k, ties=ties)
    with pc.Context(1, rows, n, 128, torch.bfloat16) as ctx:
        idx = ctx.topk(s.view(1, rows, 1, n).to(DEV), k)
        torch.cuda.synchronize()
    want = oracle.topk_columns(f64(s), k)
    assert np.array_equal(idx.cpu().numpy().reshape(rows, k), want)


@pytest.mark.parametrize("n", [4096, 5001])
def test_topk_orders_signs_magnitudes_and_narrow_ranges(n):
    """Rows whose keys differ in the sign bit, in the exponent, or only in the last mantissa bits
    (the radix select starts at the highest bit that differs inside the row); n = 5001 takes the
    streaming kernel, n = 4096 the register-resident one."""
    say(f"topk value ranges n={n}")
    g = torch.Generator().manual_seed(n)
    s = torch.empty(6, n)
    s[0] = torch.randn(n, generator=g)                                      # both signs
    s[1] = -torch.rand(n, generator=g) - 1.0                                # all negative
    s[2] = torch.rand(n, generator=g) * 1e30                                # huge
    s[3] = 1.0 + torch.randint(0, 7, (n,), generator=g).float() * 2.0 ** -23    # differ in 3 mantissa bits: many ties
    s[4] = torch.randn(n, generator=g) * 10.0 ** torch.randint(-30, 30, (n,), generator=g).float()   # every exponent
    s[5] = torch.where(torch.rand(n, generator=g) < 0.5, torch.tensor(0.0), torch.rand(n, generator=g))  # half zeros (+0)
    for k in (1, 7, n // 3, n - 1, n):
        with pc.Context(1, 6, n, 128, torch.bfloat16) as ctx:
            idx = ctx.topk(s.view(1, 6, 1, n).to(DEV), k).cpu().numpy().reshape(6, k)
        assert np.array_equal(idx, oracle.topk_columns(f64(s), k)), f"k={k}"


@pytest.mark.parametrize("rows,n,k", [(777, 4096, 409), (600, 16384, 1638), (520, 65536, 6553)])
def test_topk_rows_of_changing_distributions(rows, n, k):
    """A workgroup walks over consecutive rows and starts each select from a bracket around the threshold of
    the row before.  Consecutive rows here differ in scale, sign, spread and number of ties, so the bracket
    misses on either side, overflows, or holds the answer among ties: every row must still be exact."""
    say(f"topk changing rows={rows} n={n} k={k}")
    g = torch.Generator().manual_seed(rows + n)
    s = torch.rand(rows, n, generator=g) / n
    kind = torch.arange(rows) % 9
    s[kind == 1] *= 1000.0                                                         # threshold far above the last one
    s[kind == 2] *= 1e-3                                                           # far below
    s[kind == 3] = 1.0 + torch.randint(0, 5, (int((kind == 3).sum()), n), generator=g).float() * 2.0 ** -23   # a few values, many ties
    s[kind == 4] = -s[kind == 4]                                                   # negative
    s[kind == 5] = 0.25                                                            # all equal
    s[kind == 6] = s[kind == 6] * (1.0 + 1e-6 * torch.randn(int((kind == 6).sum()), 1, generator=g))   # like the row before the break
    s[kind == 7] = torch.round(s[kind == 7] * n * 64.0) / (n * 64.0)              # 65 levels: the threshold is a tie
    # kind 0 and 8: plain rows next to each other (the bracket holds)
    with pc.Context(1, rows, n, 128, torch.bfloat16) as ctx:
        idx = ctx.topk(s.view(1, rows, 1, n).to(DEV), k)
        again = ctx.topk(s.view(1, rows, 1, n).to(DEV), k)
        torch.cuda.synchronize()
    assert torch.equal(idx, again)
    want = oracle.topk_columns(f64(s), k)
    got = idx.cpu().numpy().reshape(rows, k)
    bad = np.nonzero((got != want).any(axis=1))[0]
    assert bad.size == 0, f"rows {bad[:8].tolist()} (kinds {kind[bad[:8]].tolist()}) differ"


def test_topk_degenerate_rows():
    n = 3000
    say("topk degenerate rows")
    s = torch.zeros(3, n)
    s[0] = 0.125                                   # all equal -> lowest indices
    s[1, 100:110] = 1.0                            # k larger than the number of non-zeros
    s[2] = torch.arange(n, dtype=torch.float32)    # strictly increasing -> the last k
    with pc.Context(1, 3, n, 128, torch.bfloat16) as ctx:
        idx = ctx.topk(s.view(1, 3, 1, n).to(DEV), 25).cpu().numpy().reshape(3, 25)
    assert np.array_equal(idx, oracle.topk_columns(f64(s), 25))
    assert idx[0].tolist() == list(range(25))
    assert idx[1].tolist() == list(range(15)) + list(range(100, 110))
    assert idx[2].tolist() == list(range(n - 25, n))


def test_tiny_workload_select_then_attn():
    w = wl.WORKLOADS["tiny"]
    say("tiny workload")
    Q, K, V = wl.make_qkv(w)
    keep = w.keep_ratios[0]
    with pc.Context(w.batch, w.heads, w.seq, w.head_dim, w.torch_dtype) as ctx:
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        idx = ctx.select(q, k_, keep)
        idx_again = ctx.select(None, None, keep, refresh=False)
        torch.cuda.synchronize()
        assert torch.equal(idx, idx_again)
        k = oracle.num_keep(w.seq, keep)
        assert idx.shape == (1, w.heads, 1, k)
        for h in range(w.heads):
            s64 = oracle.column_scores(f64(Q[0, h]), f64(K[0, h]))[0]
            assert_idx_matches(idx[0, h, 0].cpu().numpy(), s64, k, f"tiny head {h}")
            assert set(wl.heavy_columns(w, 0, h).tolist()) <= set(idx[0, h, 0].tolist())
        # attention through the ORACLE's column sets (no oracle input comes from the GPU)
        oidx = np.stack([oracle.select_columns(f64(Q[0, h]), f64(K[0, h]), keep) for h in range(w.heads)])
        O = ctx.attn(q, k_, v, torch.from_numpy(oidx).to(torch.int32).view(1, w.heads, 1, k).to(DEV))
        torch.cuda.synchronize()
    for h in range(w.heads):
        want = oracle.sparse_attention_masked(f64(Q[0, h]), f64(K[0, h]), f64(V[0, h]), oidx[h])
        assert_close(O[0, h], want, "f32", f"tiny attn head {h}")


@pytest.mark.parametrize("n,d,dtype,keep", [(1200, 128, torch.bfloat16, 0.1), (900, 64, torch.bfloat16, 0.3),
                                            (500, 128, torch.float32, 0.2)])
def test_select_near_tie_rule(n, d, dtype, keep):
    B, H = 1, 4
    say(f"select case n={n} d={d} {dtype} keep={keep}")
    Q, K, _ = rand_qkv(B, H, n, d, dtype, seed=4000 + n)
    K[:, :, 5::13] *= 2.5
    with pc.Context(B, H, n, d, dtype) as ctx:
        idx = ctx.select(Q.to(DEV), K.to(DEV), keep)
        torch.cuda.synchronize()
    k = oracle.num_keep(n, keep)
    for h in range(H):
        s64 = oracle.column_scores(f64(Q[0, h]), f64(K[0, h]))[0]
        assert_idx_matches(idx[0, h, 0].cpu().numpy(), s64, k, f"select head {h}")


# ---------------------------------------------------------------------------------------
# error paths that need a live context
# ---------------------------------------------------------------------------------------
def test_error_paths_on_device():
    say("error paths")
    B, H, n, d = 1, 2, 256, 128
    Q, K, V = (t.to(DEV) for t in rand_qkv(B, H, n, d, torch.bfloat16, seed=71))
    idx = random_idx(n, 32, B * H, seed=72).view(B, H, 1, 32).to(DEV)
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx:
        with pytest.raises(pc.PulseColError) as e:
            ctx.select(None, None, 0.1, refresh=False)
        assert e.value.status == pc.ERR_NO_PATTERN
        ctx.select(Q, K, 0.1)
        with pytest.raises(pc.PulseColError) as e:
            ctx.select(None, None, 0.2, refresh=False)          # cached k differs
        assert e.value.status == pc.ERR_NO_PATTERN
        with pytest.raises(pc.PulseColError) as e:
            ctx.select(Q, K, 1.5)
        assert e.value.status == pc.ERR_INVALID_ARG
        L = pc.lib()
        st = L.pulsecol_attn(ctx._h, Q.data_ptr() + 2, K.data_ptr(), V.data_ptr(), idx.data_ptr(), 32, Q.data_ptr(), None)
        assert st == pc.ERR_ALIGNMENT
        st = L.pulsecol_attn(ctx._h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), idx.data_ptr(), n + 1, Q.data_ptr(), None)
        assert st == pc.ERR_INVALID_ARG
        st = L.pulsecol_attn(ctx._h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), None, 32, Q.data_ptr(), None)
        assert st == pc.ERR_INVALID_ARG
        assert "idx" in pc.last_error(ctx._h)
        st = L.pulsecol_topk(ctx._h, None, 3, idx.data_ptr(), None)
        assert st == pc.ERR_INVALID_ARG
        # the context still works after failures
        O = ctx.attn(Q, K, V, idx)
        torch.cuda.synchronize()
        assert torch.isfinite(O.float()).all()
    with pytest.raises(pc.PulseColError):
        pc.Context(1, 2, 256, 128, torch.bfloat16, device=99)
    # a cache sized for keep <= 0.25: larger ratios are refused, smaller ones select and reuse as usual
    with pc.Context(B, H, n, d, torch.bfloat16, max_keep_ratio=0.25) as small, pc.Context(B, H, n, d, torch.bfloat16) as full:
        with pytest.raises(pc.PulseColError) as e:
            small.select(Q, K, 0.5)
        assert e.value.status == pc.ERR_INVALID_ARG and "max_keep_ratio" in str(e.value)
        with pytest.raises(pc.PulseColError) as e:
            small.refresh_dense(Q, K, V, 0.26)
        assert e.value.status == pc.ERR_INVALID_ARG
        a = small.select(Q, K, 0.25)
        b = small.select(None, None, 0.25, refresh=False)
        c = full.select(Q, K, 0.25)
        torch.cuda.synchronize()
        assert torch.equal(a, b) and torch.equal(a, c)


# ---------------------------------------------------------------------------------------
# refresh step that keeps the dense output
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,d,dtype,keep", [(1000, 128, torch.bfloat16, 0.1), (700, 64, torch.bfloat16, 0.2),
                                            (333, 128, torch.float32, 0.25)])
def test_refresh_dense_gives_dense_output_and_the_select_pattern(n, d, dtype, keep):
    B, H = 1, 3
    say(f"refresh_dense case n={n} d={d} {dtype} keep={keep}")
    Q, K, V = rand_qkv(B, H, n, d, dtype, seed=8000 + n)
    K[:, :, 3::11] *= 2.5
    k = oracle.num_keep(n, keep)
    with pc.Context(B, H, n, d, dtype) as ctx:
        q, k_, v = Q.to(DEV), K.to(DEV), V.to(DEV)
        O, idx = ctx.refresh_dense(q, k_, v, keep)
        cached = ctx.select(None, None, keep, refresh=False)
        Od = ctx.attn_dense(q, k_, v)
        torch.cuda.synchronize()
    assert torch.equal(O, Od)                   # the same kernel with one more output
    assert torch.equal(idx, cached)             # the pattern is cached like select's
    for h in range(H):
        qh, kh, vh = f64(Q[0, h]), f64(K[0, h]), f64(V[0, h])
        assert_close(O[0, h], oracle.dense_attention(qh, kh, vh), kind_of(dtype), f"refresh_dense O head {h}")
        assert_idx_matches(idx[0, h, 0].cpu().numpy(), oracle.column_scores(qh, kh)[0], k, f"refresh_dense idx head {h}")


def test_validation_mode_rejects_out_of_range_columns():
    """With validation on, an out-of-range column number is reported and nothing is launched
    (the output buffer keeps its contents); valid sets give the same output as without it."""
    say("validation mode")
    B, H, n, d, k = 1, 2, 512, 128, 40
    Q, K, V = (t.to(DEV) for t in rand_qkv(B, H, n, d, torch.bfloat16, seed=81))
    good = random_idx(n, k, B * H, seed=82).view(B, H, 1, k).to(DEV)
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx:
        want = ctx.attn(Q, K, V, good).clone()
        ctx.set_validation(True)
        assert torch.equal(ctx.attn(Q, K, V, good), want)
        for bad_value in (n, -1, 2**31 - 1):
            bad = good.clone()
            bad[0, 1, 0, 17] = bad_value
            O = torch.full_like(Q, 3.0)
            with pytest.raises(pc.PulseColError) as e:
                ctx.attn(Q, K, V, bad, O=O)
            assert e.value.status == pc.ERR_BAD_INDEX
            torch.cuda.synchronize()
            assert bool((O == 3.0).all())
        ctx.set_validation(False)
        assert torch.equal(ctx.attn(Q, K, V, good), want)
        torch.cuda.synchronize()


# ---------------------------------------------------------------------------------------
# work distribution of the bf16 attention kernels
# ---------------------------------------------------------------------------------------
def test_two_contexts_on_two_streams_at_once():
    """Calls on different contexts may overlap in time (each context owns its scratch and its
    work counters): two streams of default priority, each running select + attention launches of
    its own context back to back, give what the same calls give one after the other."""
    B, H, n, d, k = 1, 4, 2048, 128, 300
    say("two contexts, two streams")
    inputs = []
    for seed in (91, 92):
        Q, K, V = rand_qkv(B, H, n, d, torch.bfloat16, seed=seed)
        idx = random_idx(n, k, B * H, seed=seed + 10).view(B, H, 1, k)
        inputs.append(tuple(t.to(DEV) for t in (Q, K, V, idx)))
    with pc.Context(B, H, n, d, torch.bfloat16) as c0, pc.Context(B, H, n, d, torch.bfloat16) as c1:
        ctxs = (c0, c1)
        want = []
        for c, (Q, K, V, idx) in zip(ctxs, inputs):
            want.append((c.attn(Q, K, V, idx).clone(), c.select(Q, K, 0.1, refresh=True).clone(), c.attn_dense(Q, K, V).clone()))
        torch.cuda.synchronize()
        streams = (torch.cuda.Stream(), torch.cuda.Stream())
        got = [None, None]
        for rep in range(3):
            outs = [[], []]
            for i in range(2):                       # interleaved submission: the launches of the two contexts overlap
                with torch.cuda.stream(streams[i]):
                    Q, K, V, idx = inputs[i]
                    outs[i].append(ctxs[i].attn(Q, K, V, idx))
                    outs[i].append(ctxs[i].select(Q, K, 0.1, refresh=True))
                    outs[i].append(ctxs[i].attn_dense(Q, K, V))
            for st in streams:
                st.synchronize()
            got = outs
            for i in range(2):
                for a, b in zip(got[i], want[i]):
                    assert torch.equal(a, b), f"context {i}, repetition {rep}"


def test_non_finite_inputs_stay_inside_their_head():
    """NaN / Inf in the inputs give an undefined result for the head that holds them, and
    nothing else: every call returns, the other head's outputs and columns are bit-identical
    to those of a run on clean inputs (no address, loop bound or wait depends on a value)."""
    B, H, n, d, k = 1, 2, 900, 128, 300
    say("non-finite inputs")
    Q, K, V = rand_qkv(B, H, n, d, torch.bfloat16, seed=77)
    idx = random_idx(n, k, B * H, seed=78).view(B, H, 1, k)
    Qb, Kb, Vb = Q.clone(), K.clone(), V.clone()
    Qb[0, 0, 5, 3] = float("nan")
    Qb[0, 0, 300] = float("inf")
    Kb[0, 0, 17, :] = float("-inf")
    Kb[0, 0, 400, 1] = float("nan")
    Vb[0, 0, 33, 0] = float("inf")
    with pc.Context(B, H, n, d, torch.bfloat16) as ctx:
        clean = [ctx.attn(Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV)), ctx.attn_dense(Q.to(DEV), K.to(DEV), V.to(DEV)),
                 ctx.scores(Q.to(DEV), K.to(DEV)), ctx.select(Q.to(DEV), K.to(DEV), 0.2, refresh=True)]
        dirty = [ctx.attn(Qb.to(DEV), Kb.to(DEV), Vb.to(DEV), idx.to(DEV)), ctx.attn_dense(Qb.to(DEV), Kb.to(DEV), Vb.to(DEV)),
                 ctx.scores(Qb.to(DEV), Kb.to(DEV)), ctx.select(Qb.to(DEV), Kb.to(DEV), 0.2, refresh=True)]
        torch.cuda.synchronize()
    for c, x in zip(clean, dirty):
        assert torch.equal(c[0, 1], x[0, 1])
    sel = dirty[3][0, 0, 0].cpu().numpy()          # the disturbed head still gets k distinct ascending columns in range
    assert sel.shape == (pc.num_keep(n, 0.2),) and (sel[1:] > sel[:-1]).all() and sel[0] >= 0 and sel[-1] < n


@pytest.mark.parametrize("B,H,n,k", [(1, 1, 1300, 333), (1, 5, 2100, 257), (2, 13, 700, 64), (1, 32, 1024, 128)])
def test_query_block_queues_hand_out_every_block_once(B, H, n, k):
    """The kernels' workgroups take query blocks from per-XCD queues (and from other queues once
    theirs is empty) and leave the counters at zero.  Fewer heads than queues, head counts that
    are no multiple of eight, more blocks than workgroups: every query row must come out, the
    same on every launch, with two contexts taking turns."""
    say(f"queue case B={B} H={H} n={n} k={k}")
    d = 128
    Q, K, V = rand_qkv(B, H, n, d, torch.bfloat16, seed=9000 + H * n)
    idx = random_idx(n, k, B * H, seed=77 + H).view(B, H, 1, k)
    q, k_, v, ix = Q.to(DEV), K.to(DEV), V.to(DEV), idx.to(DEV)
    with pc.Context(B, H, n, d, torch.bfloat16) as c1, pc.Context(B, H, n, d, torch.bfloat16) as c2:
        outs = []
        for rep in range(6):
            ctx = c1 if rep % 2 == 0 else c2
            O = torch.full((B, H, n, d), float("nan"), dtype=torch.bfloat16, device=DEV)
            ctx.attn(q, k_, v, ix, O)
            outs.append(O)
            if rep == 2:
                ctx.attn_dense(q, k_, v)                 # another kernel of the same family in between
                ctx.scores(q, k_)                        # and the row pass (two workgroups per CU)
        torch.cuda.synchronize()
    for O in outs:
        assert not torch.isnan(O.float()).any()          # no block left out
        assert torch.equal(O, outs[0])
    for b in range(B):
        for h in range(0, H, max(1, H // 3)):
            want = oracle.sparse_attention_masked(f64(Q[b, h]), f64(K[b, h]), f64(V[b, h]), idx[b, h].numpy())
            assert_close(outs[-1][b, h], want, "bf16", f"queues b{b} h{h}")
