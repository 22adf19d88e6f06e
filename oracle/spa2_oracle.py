"""Plain fp64 CPU oracle for the SpargeAttention2 hot path.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the smoke
entry and the benchmark's ``cpu_baseline`` leg may import it.  It shares no
code, table or helper with the HIP library and never imports it; the HIP
library never imports this.  Everything is numpy in float64, written so that a
reader can check it against the paper by eye: no tiling, no fusion, no tricks.

What is computed (per batch element and head, independently):

* block partition, Sec. 2.1 / Alg. 1 steps 2-3:  T_m = ceil(N / b_q) query
  blocks, T_n = ceil(N / b_kv) key/value blocks (ceil, because the video token
  counts are not multiples of the block sizes; the last block is short);
* mean pooling and the pooled attention map, Sec. 2.2 and Alg. 1 step 4:
  Qbar, Kbar, Sbar = Qbar Kbar^T / sqrt(d), Pbar = row-softmax(Sbar);
* Top-k, Top-p (Sec. 2.2) and their union (Sec. 4.1 equation, Alg. 1 steps
  5-6) giving the block mask Mbar;
* block-sparse attention: the masked, renormalised softmax of Sec. 3.1
  (o_s = (p (.) m / tau) V), which is what the recurrence of Alg. 1 steps 7-21
  evaluates; written three ways (definition, per-block gather, and tile by
  tile with a final merge) that the tests cross-check;
* gradients of that map w.r.t. Q, K, V with the mask held constant (the paper
  only says a backward pass exists, Sec. 4.3; this is ordinary softmax
  calculus);
* the velocity distillation loss of Sec. 4.2 and its gradient.

Readings taken where the paper is silent are listed in the repository's design
notes; the ones that matter here:
  - ties in Pbar are ordered by lower block index first;
  - Top-p stops at the first prefix whose sum is >= p (the "at least p" of
    Sec. 2.2; the sink example of Case 1 needs >=, not >);
  - k is turned into a block count once, by `topk_blocks`;
  - every row keeps at least one block;
  - a short last block is pooled over its valid tokens only and counts as one
    block in Pbar.

Parity pins (tests/test_oracle_*.py): the paper's worked examples (Case 1's
ten-times-0.1 row and sink row, Case 2's dropped-mass example), the error
decomposition of Sec. 3.1, brute-force set union vs. prefix form, closed forms
for pooling / uniform Pbar, torch's fp64 scaled_dot_product_attention and
autograd for the full mask, finite differences for the gradients.
Tables 1-6 of the paper need matrices, weights or datasets that are not
available: parity unpinned for those numbers (nothing here depends on them).
"""
from __future__ import annotations

import math

import numpy as np

BQ = 128   # b_q,  App. A "Sparse Attention Settings"
BKV = 64   # b_kv, App. A "Sparse Attention Settings"


# --------------------------------------------------------------------------
# Block partition (Sec. 2.1; Alg. 1 steps 2-3)
# --------------------------------------------------------------------------
def num_blocks(n_tokens: int, block: int) -> int:
    return -(-int(n_tokens) // int(block))


def topk_blocks(k_frac: float, t_n: int) -> int:
    """Number of blocks "the k% largest positions" (Sec. 2.2, Top-k) means for a
    row of t_n blocks: ceil(k * t_n), at least 1 when k > 0, 0 when k == 0
    (Top-p-only mode).  The 1e-9 guards products such as 0.2 * 10 that are
    integral in exact arithmetic (Case 1: Top-20% of ten entries keeps two)."""
    if k_frac <= 0.0:
        return 0
    return int(min(t_n, max(1, math.ceil(k_frac * t_n - 1e-9))))


# --------------------------------------------------------------------------
# Pooling and the pooled attention map (Sec. 2.2; Alg. 1 step 4)
# --------------------------------------------------------------------------
def pool(x: np.ndarray, block: int) -> np.ndarray:
    """Mean over the tokens of each block.  x: [N, d] -> [ceil(N/block), d]."""
    x = np.asarray(x, dtype=np.float64)
    n, d = x.shape
    t = num_blocks(n, block)
    out = np.empty((t, d), dtype=np.float64)
    for b in range(t):
        rows = x[b * block:min(n, (b + 1) * block)]
        out[b] = rows.sum(axis=0) / rows.shape[0]
    return out


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def pooled_map(q: np.ndarray, k: np.ndarray, scale: float | None = None,
               bq: int = BQ, bkv: int = BKV) -> np.ndarray:
    """Pbar = softmax(pool(Q) pool(K)^T * scale), scale = 1/sqrt(d) by default."""
    d = q.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    qbar = pool(q, bq)
    kbar = pool(k, bkv)
    sbar = (qbar @ kbar.T) * scale
    return softmax_rows(sbar)


# --------------------------------------------------------------------------
# Top-k, Top-p and the hybrid rule (Sec. 2.2; Sec. 4.1; Alg. 1 steps 5-6)
# --------------------------------------------------------------------------
def descending_order(p_row: np.ndarray) -> np.ndarray:
    """Indices of p_row sorted by value descending, equal values by lower index
    first (a strict total order)."""
    p_row = np.asarray(p_row, dtype=np.float64)
    idx = np.arange(p_row.shape[0])
    # lexsort: last key is the primary one
    return np.lexsort((idx, -p_row))


def topk_set(p_row: np.ndarray, k_cnt: int) -> set:
    """Top-k(Pbar_i, k%): the k_cnt largest positions of the row."""
    order = descending_order(p_row)
    return set(int(j) for j in order[:k_cnt])


def topp_set(p_row: np.ndarray, top_p: float) -> set:
    """Top-p(Pbar_i, p%): the minimal prefix of the descending order whose
    summed probability is at least p (empty when p == 0)."""
    order = descending_order(p_row)
    chosen = set()
    total = 0.0
    for j in order:
        if total >= top_p:
            break
        chosen.add(int(j))
        total += float(p_row[j])
    return chosen


def hybrid_mask_bruteforce(pbar: np.ndarray, k_cnt: int, top_p: float) -> np.ndarray:
    """The equation of Sec. 4.1 taken literally: Mbar_ij = 1 iff j is in
    Top-k(row i) UNION Top-p(row i).  Pure Python sets; for small inputs."""
    t_m, t_n = pbar.shape
    m = np.zeros((t_m, t_n), dtype=np.uint8)
    for i in range(t_m):
        keep = topk_set(pbar[i], k_cnt) | topp_set(pbar[i], top_p)
        if not keep:                       # every row keeps at least one block
            keep = {int(descending_order(pbar[i])[0])}
        for j in keep:
            m[i, j] = 1
    return m


def prefix_lengths(pbar: np.ndarray, k_cnt: int, top_p: float):
    """Per row: the descending order, n_p (Top-p prefix length) and
    n = min(T_n, max(1, k_cnt, n_p)).  Both rules pick prefixes of the same
    order, so their union is the longer prefix."""
    pbar = np.asarray(pbar, dtype=np.float64)
    t_m, t_n = pbar.shape
    idx = np.broadcast_to(np.arange(t_n), pbar.shape)
    order = np.lexsort((idx, -pbar), axis=-1)
    sorted_p = np.take_along_axis(pbar, order, axis=-1)
    csum = np.cumsum(sorted_p, axis=-1)          # sequential, in sorted order
    # n_p = smallest n >= 0 with (sum of the first n) >= p
    reached = csum >= top_p
    first = np.where(reached.any(axis=-1), reached.argmax(axis=-1) + 1, t_n)
    n_p = np.where(top_p <= 0.0, 0, first)
    n = np.minimum(t_n, np.maximum(np.maximum(1, k_cnt), n_p))
    return order, n_p.astype(np.int64), n.astype(np.int64), csum


def hybrid_mask(pbar: np.ndarray, k_cnt: int, top_p: float) -> np.ndarray:
    """Mbar = Top-kp(Pbar, k%, p%) in prefix form (vectorised over rows)."""
    order, _, n, _ = prefix_lengths(pbar, k_cnt, top_p)
    t_m, t_n = pbar.shape
    rank = np.empty_like(order)
    np.put_along_axis(rank, order, np.broadcast_to(np.arange(t_n), order.shape), axis=-1)
    return (rank < n[:, None]).astype(np.uint8)


def block_mask(q, k, k_cnt: int, top_p: float, scale: float | None = None,
               bq: int = BQ, bkv: int = BKV):
    """Alg. 1 steps 2-6 for one head.  Returns (Mbar uint8 [T_m,T_n], Pbar)."""
    pbar = pooled_map(q, k, scale, bq, bkv)
    return hybrid_mask(pbar, k_cnt, top_p), pbar


# --------------------------------------------------------------------------
# Block-sparse attention forward
# --------------------------------------------------------------------------
def expand_mask(mbar: np.ndarray, n: int, bq: int = BQ, bkv: int = BKV) -> np.ndarray:
    """Token-level mask M [N,N] that is constant on each tile (Sec. 2.1)."""
    return np.repeat(np.repeat(np.asarray(mbar) != 0, bq, axis=0), bkv, axis=1)[:n, :n]


def attention_definition(q, k, v, mbar, scale: float | None = None,
                         bq: int = BQ, bkv: int = BKV):
    """Masked, renormalised softmax attention written out (Sec. 2.1, Sec. 3.1):
    S = Q K^T * scale, masked entries removed from numerator and denominator,
    O = P V.  Returns (O [N,d], LSE [N], P [N,N]).  O(N^2) memory: small N only."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    n, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    s = (q @ k.T) * scale
    keep = expand_mask(mbar, n, bq, bkv)
    s = np.where(keep, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    p = e / l
    return p @ v, (m + np.log(l))[:, 0], p


def attention_gather(q, k, v, mbar, scale: float | None = None,
                     bq: int = BQ, bkv: int = BKV, q_blocks=None):
    """Same map, evaluated per query block on the gathered selected K/V blocks
    only (exact, not an approximation; this is the form that scales to long
    sequences).  Returns (O [N,d], LSE [N]).  With `q_blocks` (an iterable of
    query-block indices) only those blocks are evaluated and the other rows of
    the outputs stay zero: used to spot-check very long sequences."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    n, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    o = np.zeros((n, d), np.float64)
    lse = np.zeros((n,), np.float64)
    for i in (range(mbar.shape[0]) if q_blocks is None else q_blocks):
        r0, r1 = i * bq, min(n, (i + 1) * bq)
        cols = np.concatenate([np.arange(j * bkv, min(n, (j + 1) * bkv))
                               for j in np.flatnonzero(mbar[i])])
        s = (q[r0:r1] @ k[cols].T) * scale
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=1, keepdims=True)
        o[r0:r1] = (e / l) @ v[cols]
        lse[r0:r1] = (m + np.log(l))[:, 0]
    return o, lse


def attention_tile_merge(q, k, v, mbar, scale: float | None = None,
                         bq: int = BQ, bkv: int = BKV):
    """What the recurrence of Alg. 1 steps 7-21 computes, evaluated tile by tile WITHOUT running state: every
    selected tile (i, j) gets its own local softmax (row-wise log-sum-exp LSE_ij and normalised output O_ij over
    the 64 keys of the tile alone); the tiles of a query block are then combined in one step with the weights
    exp(LSE_ij - LSE_i), LSE_i = log sum_j exp(LSE_ij).  Step 18's final division is what makes this equal to
    the masked softmax over all selected keys.  Unselected tiles contribute nothing (Alg. 1 step 9)."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    n, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    o = np.zeros((n, d), np.float64)
    lse = np.zeros((n,), np.float64)
    t_m, t_n = mbar.shape
    for i in range(t_m):
        r0, r1 = i * bq, min(n, (i + 1) * bq)
        local_lse, local_o = [], []
        for j in range(t_n):
            if mbar[i, j] == 0:
                continue
            c0, c1 = j * bkv, min(n, (j + 1) * bkv)
            s_ij = (q[r0:r1] @ k[c0:c1].T) * scale
            top = s_ij.max(axis=1, keepdims=True)
            w_ij = np.exp(s_ij - top)
            z_ij = w_ij.sum(axis=1, keepdims=True)
            local_lse.append(top + np.log(z_ij))             # [rows, 1]
            local_o.append((w_ij / z_ij) @ v[c0:c1])         # [rows, d], normalised within the tile
        stack = np.concatenate(local_lse, axis=1)            # [rows, tiles]
        top = stack.max(axis=1, keepdims=True)
        row_lse = top + np.log(np.exp(stack - top).sum(axis=1, keepdims=True))
        weights = np.exp(stack - row_lse)                    # each row sums to 1 over the tiles
        o[r0:r1] = sum(weights[:, t:t + 1] * local_o[t] for t in range(len(local_o)))
        lse[r0:r1] = row_lse[:, 0]
    return o, lse


# --------------------------------------------------------------------------
# Backward (mask constant; gradients w.r.t. Q, K, V)
# --------------------------------------------------------------------------
def attention_bwd_definition(q, k, v, mbar, d_o, scale: float | None = None,
                             bq: int = BQ, bkv: int = BKV):
    """Gradient of attention_definition's O w.r.t. Q, K, V for upstream dO.
    With P the masked softmax:  dV = P^T dO;  dP = dO V^T;
    D_r = sum_c dO_rc O_rc;  dS = P (.) (dP - D);  dQ = dS K * scale;
    dK = dS^T Q * scale.  Returns (dQ, dK, dV)."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    d_o = np.asarray(d_o, np.float64)
    d = q.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    o, _, p = attention_definition(q, k, v, mbar, scale, bq, bkv)
    dv = p.T @ d_o
    dp = d_o @ v.T
    dd = (d_o * o).sum(axis=1, keepdims=True)
    ds = p * (dp - dd)
    return (ds @ k) * scale, (ds.T @ q) * scale, dv


def attention_bwd_gather(q, k, v, mbar, d_o, scale: float | None = None,
                         bq: int = BQ, bkv: int = BKV, q_blocks=None):
    """Same gradients, per query block on the selected K/V blocks only.
    Returns (dQ, dK, dV, O, LSE).  With `q_blocks` only those query blocks are
    visited: their rows of dQ, O, LSE are complete, and dK, dV hold the
    contributions of those blocks only (complete for a key block whose whole
    column of the mask is listed)."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    d_o = np.asarray(d_o, np.float64)
    n, d = q.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    o = np.zeros((n, d)); lse = np.zeros((n,))
    dq = np.zeros((n, d)); dk = np.zeros((n, d)); dv = np.zeros((n, d))
    for i in (range(mbar.shape[0]) if q_blocks is None else q_blocks):
        r0, r1 = i * bq, min(n, (i + 1) * bq)
        cols = np.concatenate([np.arange(j * bkv, min(n, (j + 1) * bkv))
                               for j in np.flatnonzero(mbar[i])])
        s = (q[r0:r1] @ k[cols].T) * scale
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=1, keepdims=True)
        p = e / l
        o_i = p @ v[cols]
        o[r0:r1] = o_i
        lse[r0:r1] = (m + np.log(l))[:, 0]
        do_i = d_o[r0:r1]
        dp = do_i @ v[cols].T
        dd = (do_i * o_i).sum(axis=1, keepdims=True)
        ds = p * (dp - dd)
        dq[r0:r1] = (ds @ k[cols]) * scale
        np.add.at(dk, cols, (ds.T @ q[r0:r1]) * scale)
        np.add.at(dv, cols, p.T @ do_i)
    return dq, dk, dv, o, lse


# --------------------------------------------------------------------------
# Sparse-attention error model of Sec. 3.1 (used by the pins)
# --------------------------------------------------------------------------
def error_terms(p_row, m_row, v):
    """For one attention row p (sums to 1), mask m and values V: returns
    (tau, o, o_s, dropped, renorm) with o - o_s = dropped + renorm, where
    dropped = (p (.) (1-m)) V and renorm = (1 - 1/tau) (p (.) m) V."""
    p_row = np.asarray(p_row, np.float64); m_row = np.asarray(m_row, np.float64)
    v = np.asarray(v, np.float64)
    tau = float((p_row * m_row).sum())
    o = p_row @ v
    o_s = (p_row * m_row / tau) @ v
    dropped = (p_row * (1.0 - m_row)) @ v
    renorm = (1.0 - 1.0 / tau) * ((p_row * m_row) @ v)
    return tau, o, o_s, dropped, renorm


def error_sums(q, k, v, mbar, scale: float | None = None):
    """Sec. 3.1 summed over one head: with the full attention weights P of every query row and the token-level
    mask m expanded from the block mask, returns the L1 norms (over all rows and channels) of o - o_s, of o,
    of the dropped error and of the renormalisation error, and the sum of tau over the rows.  Dense N x N
    work: small inputs only."""
    q = np.asarray(q, np.float64); k = np.asarray(k, np.float64); v = np.asarray(v, np.float64)
    n, d = q.shape
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    p = softmax_rows(q @ k.T * scale)
    m = expand_mask(mbar, n).astype(np.float64)
    tot = ref = drop = ren = tau_sum = 0.0
    for r in range(n):
        tau, o, o_s, dropped, renorm = error_terms(p[r], m[r], v)
        tot += np.abs(o - o_s).sum(); ref += np.abs(o).sum()
        drop += np.abs(dropped).sum(); ren += np.abs(renorm).sum(); tau_sum += tau
    return tot, ref, drop, ren, tau_sum


# --------------------------------------------------------------------------
# Velocity distillation loss (Sec. 4.2 equation; Alg. 2 loss step)
# --------------------------------------------------------------------------
def vd_loss(u_sparse, u_full, weight: float):
    """L_VD = weight * ||u_sparse - u_full||^2 over all elements, and its gradient with respect to the student's
    prediction, 2 * weight * (u_sparse - u_full).  The paper's expectation over training samples is
    weight = 1 / (number of samples in the batch); weight = 1 / (number of elements) is the per-element mean."""
    a = np.asarray(u_sparse, np.float64); b = np.asarray(u_full, np.float64)
    diff = a - b
    return float(weight * (diff * diff).sum()), 2.0 * weight * diff


# --------------------------------------------------------------------------
# Batched wrappers: [B, H, N, d] arrays, heads independent
# --------------------------------------------------------------------------
def block_mask_bh(q, k, k_cnt: int, top_p: float, scale: float | None = None):
    b, h = q.shape[:2]
    masks, pbars = [], []
    for bi in range(b):
        for hi in range(h):
            m, pb = block_mask(q[bi, hi], k[bi, hi], k_cnt, top_p, scale)
            masks.append(m); pbars.append(pb)
    t_m, t_n = masks[0].shape
    return (np.stack(masks).reshape(b, h, t_m, t_n), np.stack(pbars).reshape(b, h, t_m, t_n))


def attention_bh(q, k, v, mbar, scale: float | None = None):
    b, h, n, d = q.shape
    o = np.empty((b, h, n, d)); lse = np.empty((b, h, n))
    for bi in range(b):
        for hi in range(h):
            o[bi, hi], lse[bi, hi] = attention_gather(q[bi, hi], k[bi, hi], v[bi, hi], mbar[bi, hi], scale)
    return o, lse


def attention_bwd_bh(q, k, v, mbar, d_o, scale: float | None = None):
    b, h, n, d = q.shape
    dq = np.empty((b, h, n, d)); dk = np.empty((b, h, n, d)); dv = np.empty((b, h, n, d))
    o = np.empty((b, h, n, d)); lse = np.empty((b, h, n))
    for bi in range(b):
        for hi in range(h):
            dq[bi, hi], dk[bi, hi], dv[bi, hi], o[bi, hi], lse[bi, hi] = attention_bwd_gather(
                q[bi, hi], k[bi, hi], v[bi, hi], mbar[bi, hi], d_o[bi, hi], scale)
    return dq, dk, dv, o, lse
