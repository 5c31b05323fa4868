"""Pins for the CPU oracle: everything here is fixed by the paper's definitions or by
mathematics, never by the oracle's own output.

Each pin is a function of an oracle namespace ``o`` so that the mutation tests at
the bottom can run the same pins against deliberately broken copies of the oracle
(on the CPU) and confirm that every planted mistake is caught.
"""

import itertools
import json
import math
import os
import types
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle as _oracle
from oracle import pulsecol_oracle as _impl
from paper_2605_20813_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _frac(x):
    return float(Fraction(x)) if isinstance(x, str) else float(x)


def _table(rows):
    return np.array([[_frac(v) for v in r] for r in rows], dtype=np.float64)


def _closed_form():
    with open(os.path.join(GOLDEN, "closed_form_3x4.json")) as f:
        g = json.load(f)

    def coeff(c):
        if isinstance(c, list):  # ["ln", a, m] -> m * ln(a)
            return c[2] * math.log(c[1])
        return float(c)

    Q = np.array([[coeff(c) for c in r] for r in g["Q_log_coeff"]])
    return g, Q, _table(g["K"]), _table(g["V"])


def _rand(n, d, seed, nk=None):
    r = np.random.default_rng(seed)
    return r.standard_normal((n, d)), r.standard_normal((nk or n, d)), r.standard_normal((nk or n, d))


# ----------------------------------------------------------------------------
# pins (each takes the oracle namespace)
# ----------------------------------------------------------------------------
def pin_closed_form(o):
    g, Q, K, V = _closed_form()
    np.testing.assert_allclose(np.exp(o.attention_logits(Q, K)), [[3, 1, 1], [1, 7, 1], [2, 1, 1]], rtol=1e-13)
    np.testing.assert_allclose(o.row_softmax(o.attention_logits(Q, K)), _table(g["P"]), rtol=1e-13)
    np.testing.assert_allclose(o.dense_attention(Q, K, V), _table(g["dense"]), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(o.column_scores(Q, K), _table(g["scores_one_group"]), rtol=1e-13)
    np.testing.assert_allclose(o.column_scores(Q, K, group_size=2), _table(g["scores_group_size_2"]), rtol=1e-13)
    np.testing.assert_allclose(o.column_scores(Q, K, group_size=1), _table(g["P"]), rtol=1e-13)
    assert o.topk_columns(o.column_scores(Q, K), 2).tolist() == g["top2_one_group"]
    assert o.topk_columns(o.column_scores(Q, K, group_size=2), 1).tolist() == g["top1_group_size_2"]
    # the whole identification pass on the same input: budget -> k, scores, top-k
    # (0.67 * 3 = 2.01 -> k = 2; 0.34 * 3 = 1.02 -> k = 1; 221/540 > 218/540 -> column 1 alone)
    assert o.select_columns(Q, K, 0.67).tolist() == g["top2_one_group"]
    assert o.select_columns(Q, K, 0.34).tolist() == [[1]]
    assert o.select_columns(Q, K, 0.34, group_size=2).tolist() == g["top1_group_size_2"]
    assert o.select_columns(Q, K, 1.0, group_size=2).tolist() == [[0, 1, 2], [0, 1, 2]]
    for idx, key in (([[0, 1]], "sparse_idx_0_1"), ([[0, 2]], "sparse_idx_0_2")):
        want = _table(g[key])
        np.testing.assert_allclose(o.sparse_attention_masked(Q, K, V, idx), want, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(o.sparse_attention_gathered(Q, K, V, idx), want, rtol=1e-13, atol=1e-15)
        for chunk in (1, 2, 5):
            np.testing.assert_allclose(o.sparse_attention_chunked(Q, K, V, idx, chunk), want, rtol=1e-13, atol=1e-15)


def pin_dense_matches_library(o):
    # independent routine: torch's fused scaled-dot-product attention in fp64
    Q, K, V = _rand(37, 16, 1)
    want = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])[0].numpy()
    np.testing.assert_allclose(o.dense_attention(Q, K, V), want, rtol=1e-11, atol=1e-13)
    rows = [3, 0, 36]
    np.testing.assert_allclose(o.dense_attention(Q, K, V, rows=rows), want[rows], rtol=1e-11, atol=1e-13)


def pin_scores_invariants(o):
    Q, K, _ = _rand(50, 8, 2)
    for G in (0, 1, 7, 16, 50):
        s = o.column_scores(Q, K, group_size=G)
        U = 1 if G == 0 else -(-50 // G)
        assert s.shape == (U, 50)
        assert (s >= 0).all()
        np.testing.assert_allclose(s.sum(axis=1), 1.0, rtol=1e-13)     # rows of P sum to one
    # K == 0: every logit equal, P uniform, s_j = 1/n
    np.testing.assert_allclose(o.column_scores(Q, np.zeros_like(K)), np.full((1, 50), 1 / 50), rtol=1e-13)
    # one key aligned with every query and huge: takes all the mass
    Qp = np.abs(Q) + 0.1
    Kb = K.copy()
    Kb[11] = 200.0
    s = o.column_scores(Qp, Kb)
    assert s[0, 11] > 1 - 1e-9
    # slab size is a memory bound only
    np.testing.assert_allclose(o.column_scores(Q, K, row_chunk=7), o.column_scores(Q, K, row_chunk=4096), rtol=1e-14)
    # the mean over a group of the single-row scores is the group score
    rows = o.column_scores(Q, K, group_size=1)
    np.testing.assert_allclose(o.column_scores(Q, K, group_size=7)[2], rows[14:21].mean(axis=0), rtol=1e-13)


def pin_topk_bruteforce(o):
    # Eq. 7: the chosen set maximises the captured mass over ALL subsets of size k
    for seed, n, k, G in ((3, 8, 3, 0), (4, 10, 4, 5), (5, 12, 5, 0), (6, 9, 1, 3), (7, 7, 7, 0)):
        Q, K, _ = _rand(n, 4, seed)
        s = o.column_scores(Q, K, group_size=G)
        idx = o.topk_columns(s, k)
        groups = [(0, n)] if G == 0 else [(lo, min(n, lo + G)) for lo in range(0, n, G)]
        for u, (lo, hi) in enumerate(groups):
            P = o.row_softmax(o.attention_logits(Q[lo:hi], K))
            best = max(P[:, list(C)].sum() for C in itertools.combinations(range(n), k))
            got = P[:, idx[u]].sum()
            assert got == pytest.approx(best, rel=1e-13)
            assert len(set(idx[u].tolist())) == k and list(idx[u]) == sorted(idx[u])


def pin_topk_order_and_ties(o):
    r = np.random.default_rng(8)
    s = r.random((3, 200))
    idx = o.topk_columns(s, 17)
    for u in range(3):
        want = sorted(sorted(range(200), key=lambda j: -s[u, j])[:17])
        assert idx[u].tolist() == want
    assert o.topk_columns(np.full((1, 9), 0.25), 4).tolist() == [[0, 1, 2, 3]]       # all equal -> lowest indices
    t = np.array([[0.1, 0.5, 0.3, 0.5, 0.3, 0.3, 0.9]])
    assert o.topk_columns(t, 1).tolist() == [[6]]
    assert o.topk_columns(t, 2).tolist() == [[1, 6]]                                   # tie at 0.5: index 1 before 3
    assert o.topk_columns(t, 4).tolist() == [[1, 2, 3, 6]]                             # tie at 0.3: index 2 first
    assert o.topk_columns(t, 5).tolist() == [[1, 2, 3, 4, 6]]
    assert o.topk_columns(t, 7).tolist() == [[0, 1, 2, 3, 4, 5, 6]]


def pin_sparse_attention_properties(o):
    n, d = 45, 8
    Q, K, V = _rand(n, d, 9)
    r = np.random.default_rng(10)
    idx = np.sort(r.permutation(n)[:13])[None]
    ref = o.sparse_attention_masked(Q, K, V, idx)
    # masked form == gathered form, whole or in pieces of any size (ragged last piece included)
    np.testing.assert_allclose(o.sparse_attention_gathered(Q, K, V, idx), ref, rtol=1e-13, atol=1e-15)
    for chunk in (13, 4, 5, 1, 64):
        np.testing.assert_allclose(o.sparse_attention_chunked(Q, K, V, idx, chunk), ref, rtol=1e-12, atol=1e-14)
    # column order inside idx carries no meaning
    perm = idx[:, r.permutation(13)]
    np.testing.assert_allclose(o.sparse_attention_masked(Q, K, V, perm), ref, rtol=1e-13)
    np.testing.assert_allclose(o.sparse_attention_chunked(Q, K, V, perm, 4), ref, rtol=1e-12, atol=1e-14)
    # keep everything -> dense attention
    every = np.arange(n)[None]
    np.testing.assert_allclose(o.sparse_attention_masked(Q, K, V, every), o.dense_attention(Q, K, V), rtol=1e-13)
    np.testing.assert_allclose(o.sparse_attention_chunked(Q, K, V, every, 8), o.dense_attention(Q, K, V), rtol=1e-12)
    # weights of a row sum to one: V == 1 -> O == 1; rows are convex combinations of selected V rows
    np.testing.assert_allclose(o.sparse_attention_masked(Q, K, np.ones_like(V), idx), 1.0, rtol=1e-13)
    assert (ref <= V[idx[0]].max(axis=0) + 1e-12).all() and (ref >= V[idx[0]].min(axis=0) - 1e-12).all()
    # one kept column: the output IS that value row
    np.testing.assert_allclose(o.sparse_attention_masked(Q, K, V, [[29]]), np.tile(V[29], (n, 1)), rtol=1e-14)
    np.testing.assert_allclose(o.sparse_attention_chunked(Q, K, V, [[29]], 4), np.tile(V[29], (n, 1)), rtol=1e-14)
    # unselected keys and values cannot matter
    K2, V2 = K.copy(), V.copy()
    off = np.setdiff1d(np.arange(n), idx[0])
    K2[off] += 5.0
    V2[off] -= 3.0
    np.testing.assert_allclose(o.sparse_attention_masked(Q, K2, V2, idx), ref, rtol=1e-13)
    # sampled rows == the same rows of the full result
    rows = [44, 2, 17]
    np.testing.assert_allclose(o.sparse_attention_masked(Q, K, V, idx, rows=rows), ref[rows], rtol=1e-14)
    # groups: each group attends through its own row of idx
    gidx = np.stack([np.sort(r.permutation(n)[:6]) for _ in range(3)])
    got = o.sparse_attention_masked(Q, K, V, gidx, group_size=16)
    for u, (lo, hi) in enumerate(((0, 16), (16, 32), (32, 45))):
        want = o.sparse_attention_masked(Q[lo:hi], K, V, gidx[u:u + 1])
        np.testing.assert_allclose(got[lo:hi], want, rtol=1e-13)
    np.testing.assert_allclose(o.sparse_attention_gathered(Q, K, V, gidx, group_size=16), got, rtol=1e-13)
    np.testing.assert_allclose(o.sparse_attention_chunked(Q, K, V, gidx, 4, group_size=16), got, rtol=1e-12)
    # a list counts a repeated column twice: {a, a} still yields V[a]; {a, a, b} weighs a double
    np.testing.assert_allclose(o.sparse_attention_gathered(Q, K, V, [[5, 5]]), np.tile(V[5], (n, 1)), rtol=1e-13)
    np.testing.assert_allclose(o.sparse_attention_chunked(Q, K, V, [[5, 5]], 1), np.tile(V[5], (n, 1)), rtol=1e-13)
    z = o.attention_logits(Q, K)
    w = np.exp(z[:, [5, 5, 9]])
    want = (w / w.sum(1, keepdims=True)) @ V[[5, 5, 9]]
    np.testing.assert_allclose(o.sparse_attention_gathered(Q, K, V, [[5, 5, 9]]), want, rtol=1e-12)
    np.testing.assert_allclose(o.sparse_attention_chunked(Q, K, V, [[5, 5, 9]], 2), want, rtol=1e-12)


def pin_scale_override(o):
    Q, K, V = _rand(20, 16, 11)
    np.testing.assert_allclose(o.attention_logits(Q, K), (Q @ K.T) / 4.0, rtol=1e-14)
    np.testing.assert_allclose(o.attention_logits(Q, K, scale=0.3), (Q @ K.T) * 0.3, rtol=1e-14)
    idx = np.arange(0, 20, 3)[None]
    a = o.sparse_attention_masked(Q, K, V, idx, scale=0.3)
    b = o.sparse_attention_masked(Q * 0.3 * 4.0, K, V, idx)
    np.testing.assert_allclose(a, b, rtol=1e-12)


def pin_num_keep(o):
    assert [o.num_keep(n, r) for n, r in ((256, .25), (4096, .1), (16384, .1), (32768, .05), (32768, .1),
                                           (32768, .2), (65536, .1))] == [64, 409, 1638, 1638, 3276, 6553, 6553]
    assert o.num_keep(100, 0.29) == 29          # decimal reading, not the binary product 28.999...
    assert o.num_keep(5, 0.1) == 1 and o.num_keep(7, 1.0) == 7
    for bad in ((0, .5), (8, 0.0), (8, 1.5)):
        with pytest.raises(ValueError):
            o.num_keep(*bad)


def pin_schedule(o):
    with open(os.path.join(GOLDEN, "eq8_schedules.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        assert o.refresh_schedule(c["T"], c["eta"], c["R"]) == c["tau"], c
    for T, eta, R in ((100, .5, 7), (1000, .3, 16), (17, 1.0, 17), (50, .1, 3)):
        tau = o.refresh_schedule(T, eta, R)
        T_win = max(1, math.floor(Fraction(repr(eta)) * T))
        assert len(tau) == R and tau[0] == 1 and tau[-1] == T_win
        assert all(a <= b for a, b in zip(tau, tau[1:])) and max(tau) <= T_win


def pin_schedule_variants(o):
    with open(os.path.join(GOLDEN, "schedule_variants.json")) as f:
        g = json.load(f)
    for c in g["power"]:
        assert o.refresh_schedule_power(c["T"], c["eta"], c["R"]) == c["tau"], c
    for c in g["random"]:
        assert o.refresh_schedule_random(c["T"], c["eta"], c["R"], c["uniforms"]) == c["tau"], c
    # power: same end points as the default schedule, non-decreasing, gaps that grow (refreshes
    # concentrated at the beginning of the window)
    for T, eta, R in ((1000, .3, 16), (500, .5, 9), (200, 1.0, 5)):
        tau = o.refresh_schedule_power(T, eta, R)
        uni = o.refresh_schedule(T, eta, R)
        assert len(tau) == R and tau[0] == uni[0] == 1 and tau[-1] == uni[-1]
        gaps = [b - a for a, b in zip(tau, tau[1:])]
        assert all(g >= 0 for g in gaps) and all(b >= a - 1 for a, b in zip(gaps, gaps[1:]))
        assert all(p <= u for p, u in zip(tau, uni))            # never later than the uniform placement
    # random: R distinct steps inside the window, step 1 among them; every other step of the
    # window is drawn equally often (exhaustive over a grid of uniforms on a tiny window)
    rng = np.random.default_rng(5)
    for T, eta, R in ((100, .3, 8), (64, .5, 32), (40, 1.0, 2)):
        T_win = max(1, math.floor(Fraction(repr(eta)) * T))
        tau = o.refresh_schedule_random(T, eta, R, rng.random(R - 1).tolist())
        assert len(tau) == R == len(set(tau)) and tau == sorted(tau) and tau[0] == 1 and tau[-1] <= T_win
    counts = {}
    grid = [(a + .5) / 12 for a in range(12)]
    for u0 in grid:
        for u1 in grid:
            for s_ in o.refresh_schedule_random(10, .5, 3, [u0, u1])[1:]:
                counts[s_] = counts.get(s_, 0) + 1
    assert sorted(counts) == [2, 3, 4, 5] and len(set(counts.values())) == 1
    with pytest.raises(ValueError):
        o.refresh_schedule_random(10, .3, 5, [.1, .2, .3, .4])     # window of 3 steps cannot hold 5


def pin_planted_columns_selected(o):
    w = wl.WORKLOADS["tiny"]
    for h in range(w.heads):
        q, k, _ = wl.make_head(w, 0, h)
        idx = o.select_columns(q.double().numpy(), k.double().numpy(), w.keep_ratios[0])
        heavy = set(wl.heavy_columns(w, 0, h).tolist())
        assert idx.shape == (1, 64) and heavy <= set(idx[0].tolist())


def pin_block_mask(o):
    # the block-mask equation written out as an n x n matrix, against an independent library's softmax
    n, d, kb, G = 24, 8, 4, 8
    Q, K, V = _rand(n, d, 21)
    r = np.random.default_rng(22)
    blocks = np.stack([np.sort(r.permutation(n // kb)[:2]) for _ in range(n // G)])         # G[u, c] = 1 for two blocks per query block
    S = np.zeros((n, n), dtype=bool)
    for i in range(n):
        for j in range(n):
            S[i, j] = (j // kb) in blocks[i // G]
    Z = torch.from_numpy(o.attention_logits(Q, K))
    M = torch.where(torch.from_numpy(S), 0.0, float("-inf")).double()
    want = (torch.softmax(Z + M, dim=1) @ torch.from_numpy(V)).numpy()
    np.testing.assert_allclose(o.block_sparse_attention(Q, K, V, blocks, kb, group_size=G), want, rtol=1e-12, atol=1e-14)
    assert o.block_columns([[2, 0]], 3).tolist() == [[6, 7, 8, 0, 1, 2]]
    # key blocks of one key: the column-sparse result; all key blocks kept: dense attention
    cols = np.sort(r.permutation(n)[:5])[None]
    np.testing.assert_allclose(o.block_sparse_attention(Q, K, V, cols, 1), o.sparse_attention_masked(Q, K, V, cols), rtol=1e-13)
    np.testing.assert_allclose(o.block_sparse_attention(Q, K, V, [list(range(n // kb))], kb), o.dense_attention(Q, K, V), rtol=1e-13)
    # block masses: sums of the column scores over the block's keys (each row still sums to one); blocks of
    # one key are the column scores themselves
    s = o.column_scores(Q, K, group_size=G)
    m = o.block_scores(Q, K, kb, group_size=G)
    assert m.shape == (n // G, n // kb)
    np.testing.assert_allclose(m.sum(axis=1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(m[1, 2], s[1, 8:12].sum(), rtol=1e-13)
    np.testing.assert_allclose(o.block_scores(Q, K, 1, group_size=G), s, rtol=1e-13)
    # a key block made heavy (its keys aligned with every query) must be selected; budget rule on blocks
    K2 = K.copy()
    K2[12:16] = 3.0 * Q.mean(axis=0) + 2.0
    Q2 = np.abs(Q) + 0.5
    sel = o.select_blocks(Q2, K2, 0.34, kb)              # floor(0.34 * 6) = 2 blocks
    assert sel.shape == (1, 2) and 3 in sel[0]
    assert o.select_blocks(Q, K, 0.1, kb).shape == (1, 1)
    # closed form: the 3 x 3 example with key blocks of one key, query blocks of two rows
    g, Qc, Kc, Vc = _closed_form()
    assert o.select_blocks(Qc, Kc, 0.34, 1, group_size=2).tolist() == g["top1_group_size_2"]
    np.testing.assert_allclose(o.block_sparse_attention(Qc, Kc, Vc, [[0, 1]], 1), _table(g["sparse_idx_0_1"]), rtol=1e-13, atol=1e-15)


PINS = [pin_closed_form, pin_dense_matches_library, pin_scores_invariants, pin_topk_bruteforce,
        pin_topk_order_and_ties, pin_sparse_attention_properties, pin_scale_override, pin_num_keep,
        pin_schedule, pin_schedule_variants, pin_planted_columns_selected, pin_block_mask]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(_oracle)


# ----------------------------------------------------------------------------
# mutation tests: a plausible mistake planted in a COPY of the oracle must trip a pin
# ----------------------------------------------------------------------------
def _mutant(**overrides):
    """A fresh copy of the oracle module with some functions replaced (globals rebound)."""
    src = open(_impl.__file__).read()
    mod = types.ModuleType("oracle_mutant")
    mod.__file__ = _impl.__file__
    exec(compile(src, _impl.__file__, "exec"), mod.__dict__)
    for name, fn in overrides.items():
        mod.__dict__[name] = types.FunctionType(fn.__code__, mod.__dict__, name, fn.__defaults__)
    return mod


def _logits_transposed(Q, K, scale=None):
    Q, K = _as_f64(Q), _as_f64(K)
    if scale is None:
        scale = 1.0 / math.sqrt(Q.shape[1])
    return (K @ Q.T) * scale


def _logits_no_sqrt(Q, K, scale=None):
    Q, K = _as_f64(Q), _as_f64(K)
    if scale is None:
        scale = 1.0 / Q.shape[1]
    return (Q @ K.T) * scale


def _softmax_wrong_axis(Z):
    m = np.max(Z, axis=0, keepdims=True)
    E = np.exp(Z - m)
    return E / np.sum(E, axis=0, keepdims=True)


def _softmax_no_normalise(Z):
    return np.exp(Z - np.max(Z, axis=1, keepdims=True))


def _topk_smallest(s, k):
    s = np.atleast_2d(np.asarray(s, dtype=np.float64))
    return np.stack([np.sort(np.argsort(s[u], kind="stable")[:k]) for u in range(s.shape[0])])


def _topk_high_index_ties(s, k):
    s = np.atleast_2d(np.asarray(s, dtype=np.float64))
    n = s.shape[1]
    return np.stack([np.sort((n - 1 - np.argsort(-s[u, ::-1], kind="stable"))[:k]) for u in range(s.shape[0])])


def _scores_sum_not_mean(Q, K, group_size=0, scale=None, row_chunk=2048):
    Q, K = _as_f64(Q), _as_f64(K)
    groups = _groups(Q.shape[0], group_size)
    s = np.zeros((len(groups), K.shape[0]))
    for u, (lo, hi) in enumerate(groups):
        s[u] = row_softmax(attention_logits(Q[lo:hi], K, scale)).sum(axis=0)
    return s


def _scores_divide_by_nominal_group(Q, K, group_size=0, scale=None, row_chunk=2048):
    Q, K = _as_f64(Q), _as_f64(K)
    groups = _groups(Q.shape[0], group_size)
    g = Q.shape[0] if group_size == 0 else group_size
    s = np.zeros((len(groups), K.shape[0]))
    for u, (lo, hi) in enumerate(groups):
        s[u] = row_softmax(attention_logits(Q[lo:hi], K, scale)).sum(axis=0) / g
    return s


def _scores_from_logits(Q, K, group_size=0, scale=None, row_chunk=2048):
    Q, K = _as_f64(Q), _as_f64(K)
    groups = _groups(Q.shape[0], group_size)
    s = np.zeros((len(groups), K.shape[0]))
    for u, (lo, hi) in enumerate(groups):
        s[u] = attention_logits(Q[lo:hi], K, scale).mean(axis=0)
    return s


def _schedule_zero_based(T, eta, R):
    T_win = max(1, _floor_of_product(eta, T))
    if R == 1:
        return [0]
    return [((r - 1) * (T_win - 1)) // (R - 1) for r in range(1, R + 1)]


def _schedule_window_not_minus_one(T, eta, R):
    T_win = max(1, _floor_of_product(eta, T))
    if R == 1:
        return [1]
    return [1 + ((r - 1) * T_win) // (R - 1) for r in range(1, R + 1)]


def _power_linear(T, eta, R):
    T_win = max(1, _floor_of_product(eta, T))
    if R == 1:
        return [1]
    return [1 + int(Fraction(i, R - 1) * (T_win - 1)) for i in range(R)]


def _power_whole_window(T, eta, R):
    T_win = max(1, _floor_of_product(eta, T))
    if R == 1:
        return [1]
    return [1 + int(Fraction(i * i, (R - 1) * (R - 1)) * T_win) for i in range(R)]


def _random_with_replacement(T, eta, R, uniforms):
    T_win = max(1, _floor_of_product(eta, T))
    m = T_win - 1
    if R - 1 > m:
        raise ValueError
    return sorted([1] + [2 + int(math.floor(float(u) * m)) for u in list(uniforms)[:R - 1]])


def _random_without_first_step(T, eta, R, uniforms):
    T_win = max(1, _floor_of_product(eta, T))
    pool = list(range(1, T_win + 1))
    u = [float(x) for x in uniforms] + [0.5]
    for i in range(R):
        j = i + int(math.floor(u[i] * (T_win - i)))
        pool[i], pool[j] = pool[j], pool[i]
    return sorted(pool[:R])


def _select_ignores_groups(Q, K, keep_ratio, group_size=0, scale=None):
    k = num_keep(np.asarray(Q).shape[0], keep_ratio)
    return topk_columns(column_scores(Q, K, 0, scale), k)


def _select_budget_is_sparsity(Q, K, keep_ratio, group_size=0, scale=None):
    k = num_keep(np.asarray(Q).shape[0], max(1.0 - keep_ratio, 1e-9))
    return topk_columns(column_scores(Q, K, group_size, scale), k)


def _block_columns_off_by_one(block_idx, key_block):
    blocks = np.atleast_2d(np.asarray(block_idx, dtype=np.int64))
    return (blocks[:, :, None] * key_block + 1 + np.arange(key_block)[None, None, :]).reshape(blocks.shape[0], -1) % 10**9


def _block_scores_mean_not_sum(Q, K, key_block, group_size=0, scale=None):
    s = column_scores(Q, K, group_size, scale)
    return s.reshape(s.shape[0], s.shape[1] // key_block, key_block).mean(axis=2)


def _block_scores_strided_blocks(Q, K, key_block, group_size=0, scale=None):
    s = column_scores(Q, K, group_size, scale)
    return s.reshape(s.shape[0], key_block, s.shape[1] // key_block).sum(axis=1)


def _num_keep_ceil(n, keep_ratio):
    if n < 1 or not (0.0 < keep_ratio <= 1.0):
        raise ValueError
    return max(1, math.ceil(keep_ratio * n))


MUTANTS = {
    "logits_transposed": dict(attention_logits=_logits_transposed),
    "logits_scale_1_over_d": dict(attention_logits=_logits_no_sqrt),
    "softmax_over_queries": dict(row_softmax=_softmax_wrong_axis),
    "softmax_not_normalised": dict(row_softmax=_softmax_no_normalise),
    "topk_takes_smallest": dict(topk_columns=_topk_smallest),
    "topk_ties_to_high_index": dict(topk_columns=_topk_high_index_ties),
    "scores_sum_not_mean": dict(column_scores=_scores_sum_not_mean),
    "scores_nominal_group_size": dict(column_scores=_scores_divide_by_nominal_group),
    "scores_from_raw_logits": dict(column_scores=_scores_from_logits),
    "schedule_zero_based": dict(refresh_schedule=_schedule_zero_based),
    "schedule_full_window": dict(refresh_schedule=_schedule_window_not_minus_one),
    "num_keep_ceil": dict(num_keep=_num_keep_ceil),
    "block_columns_off_by_one": dict(block_columns=_block_columns_off_by_one),
    "block_scores_mean_not_sum": dict(block_scores=_block_scores_mean_not_sum),
    "block_scores_strided_blocks": dict(block_scores=_block_scores_strided_blocks),
    "select_ignores_groups": dict(select_columns=_select_ignores_groups),
    "select_budget_is_sparsity": dict(select_columns=_select_budget_is_sparsity),
    "power_schedule_linear": dict(refresh_schedule_power=_power_linear),
    "power_schedule_whole_window": dict(refresh_schedule_power=_power_whole_window),
    "random_schedule_with_replacement": dict(refresh_schedule_random=_random_with_replacement),
    "random_schedule_without_first_step": dict(refresh_schedule_random=_random_without_first_step),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name):
    mutant = _mutant(**MUTANTS[name])
    tripped = []
    for pin in PINS:
        try:
            pin(mutant)
        except (AssertionError, ValueError, IndexError):
            tripped.append(pin.__name__)
    assert tripped, f"no pin notices the planted mistake '{name}'"


def test_chunk_merge_mistakes_are_caught():
    """The merge of partial softmax results: a dropped weight on either side, a normaliser that is
    not carried forward, or a piece normalised by the wrong sum must show."""
    src = open(_impl.__file__).read()
    for needle, broken in (("np.exp(L - L_both)[:, None] * A +", "A +"),
                           ("np.exp(L_piece - L_both)[:, None] * A_piece", "A_piece"),
                           ("L = L_both", "L = L_piece"),
                           ("L_piece = top + np.log(", "L_piece = np.log("),
                           ("A_piece = row_softmax(Z) @ V[piece]", "A_piece = np.exp(Z - top[:, None]) @ V[piece]")):
        assert needle in src
        mod = types.ModuleType("oracle_mutant")
        exec(compile(src.replace(needle, broken), "mutant", "exec"), mod.__dict__)
        with pytest.raises(AssertionError):
            pin_sparse_attention_properties(mod)
