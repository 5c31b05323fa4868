"""Plain fp64 definitions of the PulseCol attention hot path (numpy, CPU).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

Every function works on ONE attention head: ``Q, K, V`` are ``[n, d]`` float64
arrays (bf16 / fp32 inputs widened exactly by the caller, so input rounding is
not counted as error).  Column sets are ``idx[U, k]`` integer arrays, one row per
query group; ``group_size == 0`` means a single group that holds every query
(U = 1).  Nothing here is blocked, fused or reordered beyond what the cited
passage states; the only concession to memory is that independent query rows
may be processed a slab at a time (``row_chunk``), which changes no value.

Pins (tests/test_oracle_pins.py): closed-form softmax examples, the textbook
dense attention of an independent library, row-stochastic invariants, brute
force over all column subsets (Eq. 7), the masked form against the gathered form
whole and in pieces, hand-worked
refresh schedules (Eq. 8).  The paper prints no numeric example of its own, so
agreement with the authors' kernels is "parity unpinned"; agreement with the
definitions is what the pins establish.
"""

from __future__ import annotations

import math
from fractions import Fraction

import numpy as np

_F64 = np.float64


def _as_f64(x) -> np.ndarray:
    a = np.asarray(x, dtype=_F64)
    if a.ndim != 2:
        raise ValueError("expected an [n, d] array for one head")
    return a


def _floor_of_product(ratio: float, count: int) -> int:
    """floor(ratio * count) with the ratio read as the decimal the caller wrote."""
    return math.floor(Fraction(repr(float(ratio))) * int(count))


# --------------------------------------------------------------------------
# Eq. 3: sparsity budget -> number of kept columns per query row
# --------------------------------------------------------------------------
def num_keep(n: int, keep_ratio: float) -> int:
    """k = max(1, floor(keep_ratio * n)), keep_ratio = 1 - rho.

    Sec. 3.1, sparsity-budget constraint: at most (1 - rho) n^2 retained pairs
    per head, i.e. at most (1 - rho) n per query row; floor honours the "<=".
    """
    if n < 1 or not (0.0 < keep_ratio <= 1.0):
        raise ValueError("need n >= 1 and 0 < keep_ratio <= 1")
    return max(1, _floor_of_product(keep_ratio, n))


# --------------------------------------------------------------------------
# Eq. 1 and the dense attention that follows it
# --------------------------------------------------------------------------
def attention_logits(Q, K, scale: float | None = None) -> np.ndarray:
    """Z = Q K^T / sqrt(d_h)   (Sec. 3.1, logits equation).  Z[i, j] = q_i . k_j * scale."""
    Q = _as_f64(Q)
    K = _as_f64(K)
    if scale is None:
        scale = 1.0 / math.sqrt(Q.shape[1])
    return (Q @ K.T) * scale


def row_softmax(Z: np.ndarray) -> np.ndarray:
    """softmax over the key axis of each query row; -inf entries get weight 0."""
    m = np.max(Z, axis=1, keepdims=True)
    E = np.exp(Z - m)
    return E / np.sum(E, axis=1, keepdims=True)


def dense_attention(Q, K, V, scale: float | None = None, rows=None) -> np.ndarray:
    """A = softmax(Z) V   (Sec. 3.1, full bidirectional attention, no mask).

    ``rows`` (optional) restricts the result to those query rows.
    """
    Q = _as_f64(Q)
    V = _as_f64(V)
    if rows is not None:
        Q = Q[np.asarray(rows)]
    return row_softmax(attention_logits(Q, K, scale)) @ V


# --------------------------------------------------------------------------
# Eq. 5: group column scores
# --------------------------------------------------------------------------
def _groups(n: int, group_size: int):
    """Contiguous query groups G_1..G_U; group_size 0 -> one group of all rows."""
    if group_size < 0:
        raise ValueError("group_size must be >= 0")
    g = n if group_size == 0 else group_size
    return [(lo, min(n, lo + g)) for lo in range(0, n, g)]


def column_scores(Q, K, group_size: int = 0, scale: float | None = None,
                  row_chunk: int = 2048, progress=None) -> np.ndarray:
    """s[u, j] = (1/|G_u|) sum_{i in G_u} P[i, j],  P = row softmax of the FULL logits.

    Sec. 3.3, group-wise column-sparse pattern estimation (score equation).
    Returns float64 ``[U, n]``.  ``progress`` (optional) is called with the number of query
    rows done after each slab, so that long runs can report that they are alive.
    """
    Q = _as_f64(Q)
    K = _as_f64(K)
    n = Q.shape[0]
    groups = _groups(n, group_size)
    s = np.zeros((len(groups), K.shape[0]), dtype=_F64)
    for u, (lo, hi) in enumerate(groups):
        for r0 in range(lo, hi, row_chunk):
            r1 = min(hi, r0 + row_chunk)
            P = row_softmax(attention_logits(Q[r0:r1], K, scale))
            s[u] += P.sum(axis=0)
            if progress is not None:
                progress(r1)
        s[u] /= (hi - lo)
    return s


# --------------------------------------------------------------------------
# Eq. 6 / Eq. 7: top-k columns per group
# --------------------------------------------------------------------------
def topk_columns(s, k: int) -> np.ndarray:
    """C_u = TopK(s_u, k) for every row of ``s``; returns int64 ``[U, k]`` ascending.

    Sec. 3.3, TopK equation.  Equal scores: the lower column index wins (any
    maximiser of the Eq. 7 objective is correct; this fixes one).  The set is
    emitted in ascending column order; the order carries no meaning.
    """
    s = np.atleast_2d(np.asarray(s, dtype=_F64))
    U, n = s.shape
    if not (1 <= k <= n):
        raise ValueError("need 1 <= k <= n")
    out = np.empty((U, k), dtype=np.int64)
    for u in range(U):
        order = np.argsort(-s[u], kind="stable")  # score descending, index ascending on ties
        out[u] = np.sort(order[:k])
    return out


def select_columns(Q, K, keep_ratio: float, group_size: int = 0,
                   scale: float | None = None) -> np.ndarray:
    """The whole identification pass: Eq. 3 -> Eq. 5 -> Eq. 6."""
    k = num_keep(np.asarray(Q).shape[0], keep_ratio)
    return topk_columns(column_scores(Q, K, group_size, scale), k)


# --------------------------------------------------------------------------
# Eq. 2: masked sparse attention (the definition of the sparse result)
# --------------------------------------------------------------------------
def sparse_attention_masked(Q, K, V, idx, group_size: int = 0,
                            scale: float | None = None, rows=None) -> np.ndarray:
    """A~ = softmax(Z + M(S)) V with S[i, j] = 1 iff j in idx[u(i)], M = 0 / -inf.

    Sec. 3.1, masked sparse-attention equation, with the group-shared mask of
    Sec. 3.3.  ``rows`` (optional) restricts the result to those query rows.
    Column indices must be unique within a row of ``idx`` (a 0/1 mask cannot
    express multiplicity).
    """
    Q = _as_f64(Q)
    K = _as_f64(K)
    V = _as_f64(V)
    idx = np.atleast_2d(np.asarray(idx, dtype=np.int64))
    n = Q.shape[0]
    nk = K.shape[0]
    groups = _groups(n, group_size)
    if idx.shape[0] != len(groups):
        raise ValueError("idx needs one row per query group")
    row_ids = np.arange(n) if rows is None else np.asarray(rows, dtype=np.int64)
    g = n if group_size == 0 else group_size
    O = np.empty((row_ids.size, V.shape[1]), dtype=_F64)
    for u in np.unique(row_ids // g):
        sel = np.nonzero(row_ids // g == u)[0]
        M = np.full(nk, -np.inf)
        M[idx[u]] = 0.0
        Z = attention_logits(Q[row_ids[sel]], K, scale) + M[None, :]
        O[sel] = row_softmax(Z) @ V
    return O


# --------------------------------------------------------------------------
# The gathered form of the sparse result, whole and in pieces
# --------------------------------------------------------------------------
def sparse_attention_gathered(Q, K, V, idx, group_size: int = 0,
                              scale: float | None = None) -> np.ndarray:
    """Softmax over the k gathered logits of each row, applied to the gathered value rows.

    Sec. 3.4: the kernel works on K_S, V_S (the rows named by the group's column list) and
    never forms the n x n matrix.  For a list of distinct columns this equals the masked
    definition above; a column that appears twice in the list is a term twice (a 0/1 mask
    cannot say that, a list can).
    """
    Q = _as_f64(Q)
    K = _as_f64(K)
    V = _as_f64(V)
    idx = np.atleast_2d(np.asarray(idx, dtype=np.int64))
    groups = _groups(Q.shape[0], group_size)
    if idx.shape[0] != len(groups):
        raise ValueError("idx needs one row per query group")
    O = np.empty((Q.shape[0], V.shape[1]), dtype=_F64)
    for u, (lo, hi) in enumerate(groups):
        cols = idx[u]
        O[lo:hi] = row_softmax(attention_logits(Q[lo:hi], K[cols], scale)) @ V[cols]
    return O


def sparse_attention_chunked(Q, K, V, idx, chunk: int, group_size: int = 0,
                             scale: float | None = None) -> np.ndarray:
    """The gathered result built up from pieces of the column list, `chunk` entries at a time.

    This is the property the appendix algorithm "Column-Sparse Attention Forward" rests on
    (a running softmax state over tiles of the list), stated as a merge of partial results:
    a piece c of the list has, per query row, a log-normaliser L_c = log sum_t exp z_t and an
    output A_c normalised over the piece alone; two disjoint pieces a, b of a list combine to
        L = log(exp L_a + exp L_b),   A = exp(L_a - L) A_a + exp(L_b - L) A_b,
    and the result for the whole list is A after the last piece, whatever the piece size.
    """
    if chunk < 1:
        raise ValueError("chunk must be >= 1")
    Q = _as_f64(Q)
    K = _as_f64(K)
    V = _as_f64(V)
    idx = np.atleast_2d(np.asarray(idx, dtype=np.int64))
    groups = _groups(Q.shape[0], group_size)
    if idx.shape[0] != len(groups):
        raise ValueError("idx needs one row per query group")
    O = np.empty((Q.shape[0], V.shape[1]), dtype=_F64)
    for u, (lo, hi) in enumerate(groups):
        L = np.full(hi - lo, -np.inf)
        A = np.zeros((hi - lo, V.shape[1]), dtype=_F64)
        for c0 in range(0, idx.shape[1], chunk):
            piece = idx[u, c0:c0 + chunk]
            Z = attention_logits(Q[lo:hi], K[piece], scale)
            top = Z.max(axis=1)
            L_piece = top + np.log(np.exp(Z - top[:, None]).sum(axis=1))
            A_piece = row_softmax(Z) @ V[piece]
            L_both = np.logaddexp(L, L_piece)
            A = np.exp(L - L_both)[:, None] * A + np.exp(L_piece - L_both)[:, None] * A_piece
            L = L_both
        O[lo:hi] = A
    return O


# --------------------------------------------------------------------------
# Eq. 4: block-sparse attention (the formulation column sparsity is contrasted with)
# --------------------------------------------------------------------------
def block_columns(block_idx, key_block: int) -> np.ndarray:
    """The key columns of the key blocks in ``block_idx[U, kb]``: block c holds columns
    c * key_block .. (c + 1) * key_block - 1.  Returns int64 ``[U, kb * key_block]``."""
    blocks = np.atleast_2d(np.asarray(block_idx, dtype=np.int64))
    if key_block < 1:
        raise ValueError("key_block must be >= 1")
    return (blocks[:, :, None] * key_block + np.arange(key_block)[None, None, :]).reshape(blocks.shape[0], -1)


def block_sparse_attention(Q, K, V, block_idx, key_block: int, group_size: int = 0,
                           scale: float | None = None, rows=None) -> np.ndarray:
    """A~ = softmax(Z + M(S)) V with the block mask S(i, j) = G(b(i), b(j)).

    Sec. 3.1, block-mask equation: b(.) maps a position to its block, G is a 0/1 matrix over
    (query block, key block).  Query blocks are the contiguous groups of ``group_size`` rows (0: all
    rows are one block), key blocks are ``key_block`` consecutive keys; row u of ``block_idx`` lists
    the key blocks c with G[u, c] = 1.  The sequence length must be a multiple of ``key_block``.
    """
    K = _as_f64(K)
    if K.shape[0] % key_block:
        raise ValueError("the key count must be a multiple of key_block")
    return sparse_attention_masked(Q, K, V, block_columns(block_idx, key_block), group_size, scale, rows)


def block_scores(Q, K, key_block: int, group_size: int = 0, scale: float | None = None) -> np.ndarray:
    """Mass of every key block for every query group: the sum of the group's column scores (Sec. 3.3,
    score equation) over the block's keys.  Returns float64 ``[U, n / key_block]``; each row sums to 1."""
    s = column_scores(Q, K, group_size, scale)
    U, n = s.shape
    if n % key_block:
        raise ValueError("the key count must be a multiple of key_block")
    return s.reshape(U, n // key_block, key_block).sum(axis=2)


def select_blocks(Q, K, keep_ratio: float, key_block: int, group_size: int = 0,
                  scale: float | None = None) -> np.ndarray:
    """Key blocks kept under the same budget rule applied to blocks: the
    max(1, floor(keep_ratio * n / key_block)) heaviest blocks per query group, ascending."""
    n = np.asarray(K).shape[0]
    if n % key_block:
        raise ValueError("the key count must be a multiple of key_block")
    return topk_columns(block_scores(Q, K, key_block, group_size, scale), num_keep(n // key_block, keep_ratio))


# --------------------------------------------------------------------------
# Eq. 8: refresh schedule
# --------------------------------------------------------------------------
def refresh_schedule(T: int, eta: float, R: int) -> list[int]:
    """1-based refresh steps tau_1..tau_R   (Sec. 3.3, schedule equation).

    T_win = floor(eta T) (at least 1 so that tau_1 = 1 exists);
    R = 1 -> {1}; else tau_r = 1 + floor((r-1)(T_win-1)/(R-1)).
    """
    if T < 1 or R < 1 or not (0.0 < eta <= 1.0):
        raise ValueError("need T >= 1, R >= 1, 0 < eta <= 1")
    T_win = max(1, _floor_of_product(eta, T))
    if R == 1:
        return [1]
    return [1 + ((r - 1) * (T_win - 1)) // (R - 1) for r in range(1, R + 1)]


def refresh_schedule_power(T: int, eta: float, R: int) -> list[int]:
    """Power-based placement of the refresh steps (appendix, ablation on the refresh
    schedule): normalised positions (i/(R-1))^2, i = 0..R-1, inside the same early window of
    T_win = floor(eta T) steps, mapped to 1-based steps like the default schedule:
    tau_i = 1 + floor((i/(R-1))^2 (T_win-1)).  Exact rational arithmetic.
    """
    if T < 1 or R < 1 or not (0.0 < eta <= 1.0):
        raise ValueError("need T >= 1, R >= 1, 0 < eta <= 1")
    T_win = max(1, _floor_of_product(eta, T))
    if R == 1:
        return [1]
    return [1 + int(Fraction(i * i, (R - 1) * (R - 1)) * (T_win - 1)) for i in range(R)]


def refresh_schedule_random(T: int, eta: float, R: int, uniforms) -> list[int]:
    """Random placement (same appendix): R distinct refresh steps drawn uniformly from the
    window 1..T_win, returned ascending.  Step 1 always belongs to the set (a pattern must
    exist before the first sparse step); the other R-1 steps are a uniform draw without
    replacement from 2..T_win, taken from the caller's uniforms u_0..u_{R-2} in [0, 1) by a
    partial Fisher-Yates shuffle: at draw i the pool position i + floor(u_i (m - i)) is swapped
    to the front, m = T_win - 1.
    """
    if T < 1 or R < 1 or not (0.0 < eta <= 1.0):
        raise ValueError("need T >= 1, R >= 1, 0 < eta <= 1")
    T_win = max(1, _floor_of_product(eta, T))
    m = T_win - 1
    if R - 1 > m:
        raise ValueError("the window holds fewer than R steps")
    u = [float(x) for x in uniforms]
    if len(u) < R - 1 or any(not (0.0 <= x < 1.0) for x in u[:R - 1]):
        raise ValueError("need R-1 uniforms in [0, 1)")
    pool = list(range(2, T_win + 1))
    for i in range(R - 1):
        j = i + int(math.floor(u[i] * (m - i)))
        pool[i], pool[j] = pool[j], pool[i]
    return sorted([1] + pool[:R - 1])

