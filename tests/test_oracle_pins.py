"""Pins for the CPU oracle: what the paper prints, closed forms, library routines,
brute force and finite differences.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch
from hypothesis import given, settings, strategies as st
from scipy.special import softmax as scipy_softmax

from oracle import spa2_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_examples.txt")


def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, row, par, exp = [s.strip() for s in line.split("|")]
            out[name] = (np.array([float(x) for x in row.split()]), par, exp)
    return out


# ------------------------------------------------------------------ paper's worked examples
def test_case1_uniform_row_topk_keeps_two():
    row, par, exp = _golden()["caseA_topk"]
    k = float(par.split("=")[1])
    cnt = orc.topk_blocks(k, row.size)
    assert cnt == int(exp.split("=")[1]) == 2
    # all ten are tied: lower index first
    assert orc.topk_set(row, cnt) == {0, 1}
    m = orc.hybrid_mask(row[None, :], cnt, 0.0)
    assert m.tolist() == [[1, 1, 0, 0, 0, 0, 0, 0, 0, 0]]


def test_case1_sink_row_topp_keeps_only_sink():
    row, par, exp = _golden()["caseB_topp"]
    p = float(par.split("=")[1])
    assert orc.topp_set(row, p) == {int(exp.split("=")[1])} == {0}
    # Top-p alone (k=0) through the vectorised path
    assert orc.hybrid_mask(row[None, :], 0, p).tolist() == [[1, 0, 0, 0]]
    # the hybrid rule with k=50% also keeps the runner-up: union, not intersection
    assert orc.hybrid_mask(row[None, :], orc.topk_blocks(0.5, 4), p).tolist() == [[1, 1, 0, 0]]
    # strictly-greater would have taken two entries; make sure ">" is not what is implemented
    assert orc.topp_set(row, 0.6000001) == {0, 1}


@pytest.mark.parametrize("name", ["caseC_before", "caseC_after"])
def test_case2_dropped_mass_and_tau(name):
    row, par, exp = _golden()[name]
    m = np.array([float(x) for x in par.split("=")[1].split()])
    dropped_exp = np.array([float(x) for x in exp.split(";")[0].split("=")[1].split()])
    tau_exp = float(exp.split(";")[1].split("=")[1])
    v = np.eye(3)                      # V = I exposes the weight vectors themselves
    tau, o, o_s, dropped, renorm = orc.error_terms(row, m, v)
    assert tau == pytest.approx(tau_exp, abs=1e-15)
    np.testing.assert_allclose(dropped, dropped_exp, atol=1e-15)
    np.testing.assert_allclose(o - o_s, dropped + renorm, atol=1e-15)
    # and the attention routine itself produces o_s for that row: logits = log p
    q = np.ones((1, 1)); k = np.log(row)[:, None]; vv = np.eye(3)
    o_att, _, _ = orc.attention_definition(np.repeat(q, 3, 0), k, vv, np.tile(m, (3, 1)), scale=1.0, bq=1, bkv=1)
    np.testing.assert_allclose(o_att[0], o_s, atol=1e-14)


def test_topk_blocks_rule():
    assert orc.topk_blocks(0.2, 10) == 2
    assert orc.topk_blocks(0.05, 512) == 26        # 25.6 -> 26
    assert orc.topk_blocks(0.05, 1182) == 60       # 59.1 -> 60
    assert orc.topk_blocks(0.25, 32) == 8
    assert orc.topk_blocks(0.10, 512) == 52
    assert orc.topk_blocks(0.0, 512) == 0
    assert orc.topk_blocks(1e-6, 512) == 1
    assert orc.topk_blocks(1.0, 512) == 512
    assert orc.topk_blocks(3.0, 7) == 7


# ------------------------------------------------------------------ selection: brute force and invariants
probs = st.lists(st.sampled_from([0.0, 0.5, 1.0, 2.0, 3.0, 7.0]) | st.floats(0.0, 10.0), min_size=1, max_size=24)


@settings(max_examples=300, deadline=None)
@given(rows=st.lists(probs, min_size=1, max_size=4), k=st.integers(0, 30), p=st.floats(0.0, 1.0))
def test_union_of_sets_equals_longer_prefix(rows, k, p):
    t_n = max(len(r) for r in rows)
    w = np.array([r + [0.0] * (t_n - len(r)) for r in rows]) + 1e-3
    pbar = w / w.sum(axis=1, keepdims=True)
    k = min(k, t_n)
    brute = orc.hybrid_mask_bruteforce(pbar, k, p)
    fast = orc.hybrid_mask(pbar, k, p)
    assert np.array_equal(brute, fast)
    for i in range(pbar.shape[0]):
        sel = fast[i].astype(bool)
        assert sel.sum() >= max(1, k)
        assert sel.all() or pbar[i][sel].sum() >= p - 1e-12
        # superset of each rule
        for j in orc.topk_set(pbar[i], k) | orc.topp_set(pbar[i], p):
            assert sel[j]
        # selected entries dominate the rejected ones
        if not sel.all():
            assert pbar[i][sel].min() >= pbar[i][~sel].max()
        # minimality of Top-p: dropping the smallest selected entry of a Top-p-bound row falls below p
        n_p = len(orc.topp_set(pbar[i], p))
        if n_p > max(1, k):
            order = orc.descending_order(pbar[i])
            assert pbar[i][order[:n_p - 1]].sum() < p


def test_ties_break_to_lower_index_and_order_is_total():
    row = np.array([0.125, 0.25, 0.125, 0.25, 0.125, 0.125])
    assert orc.descending_order(row).tolist() == [1, 3, 0, 2, 4, 5]
    assert orc.hybrid_mask(row[None], 3, 0.0).tolist() == [[1, 1, 0, 1, 0, 0]]


def test_monotone_in_k_and_p():
    rng = np.random.default_rng(1)
    pbar = scipy_softmax(rng.normal(size=(8, 40)) * 2.0, axis=1)
    prev = None
    for k in range(0, 41, 5):
        m = orc.hybrid_mask(pbar, k, 0.3).astype(int)
        if prev is not None:
            assert (m >= prev).all()
        prev = m
    prev = None
    for p in np.linspace(0, 1, 11):
        m = orc.hybrid_mask(pbar, 4, float(p)).astype(int)
        if prev is not None:
            assert (m >= prev).all()
        prev = m
    assert orc.hybrid_mask(pbar, 0, 1.0).sum() >= 8 * 39   # p = 1 keeps (almost) everything
    assert orc.hybrid_mask(pbar, 40, 0.0).all()


def test_p_zero_is_plain_topk_and_k_zero_is_nucleus():
    rng = np.random.default_rng(2)
    pbar = scipy_softmax(rng.normal(size=(5, 33)) * 3.0, axis=1)
    m = orc.hybrid_mask(pbar, 7, 0.0)
    for i in range(5):
        top = set(np.argsort(-pbar[i], kind="stable")[:7].tolist())     # library top-k
        assert set(np.flatnonzero(m[i]).tolist()) == top
    assert (orc.prefix_lengths(pbar, 7, 0.0)[1] == 0).all()             # p = 0: the Top-p prefix is empty
    m = orc.hybrid_mask(pbar, 0, 0.7)
    for i in range(5):
        srt = np.sort(pbar[i])[::-1]
        n_p = int(np.searchsorted(np.cumsum(srt), 0.7, side="left")) + 1   # textbook nucleus size
        assert m[i].sum() == n_p


# ------------------------------------------------------------------ pooling and Pbar closed forms
def test_pool_constant_blocks_and_short_last_block():
    n, d, blk = 300, 4, 128
    x = np.zeros((n, d))
    x[:128] = 3.0; x[128:256] = -1.0; x[256:] = 5.0       # last block has 44 valid rows
    np.testing.assert_allclose(orc.pool(x, blk), [[3.0] * d, [-1.0] * d, [5.0] * d])
    # a linear ramp: block mean is the midpoint; the short block divides by its own length
    r = np.arange(n, dtype=float)[:, None] * np.ones((1, d))
    np.testing.assert_allclose(orc.pool(r, blk)[:, 0], [63.5, 191.5, (256 + 299) / 2])
    assert orc.num_blocks(32760, 128) == 256 and orc.num_blocks(32760, 64) == 512
    assert orc.num_blocks(75600, 128) == 591 and orc.num_blocks(75600, 64) == 1182


def test_pbar_uniform_when_q_is_zero_and_topp_count_closed_form():
    n, d = 1024, 8
    rng = np.random.default_rng(0)
    k = rng.normal(size=(n, d))
    pbar = orc.pooled_map(np.zeros((n, d)), k)
    t_n = n // 64
    np.testing.assert_allclose(pbar, 1.0 / t_n, rtol=0, atol=1e-16)
    np.testing.assert_allclose(pbar.sum(axis=1), 1.0, atol=1e-14)
    # uniform row: Top-p needs ceil(p * T_n) blocks (p chosen off the lattice), lowest indices first
    for p in (0.3, 0.55, 0.8):
        m = orc.hybrid_mask(pbar, 1, p)
        cnt = math.ceil(p * t_n)
        assert (m.sum(axis=1) == cnt).all()
        assert m[:, :cnt].all()


def test_pbar_rank_one_closed_form_against_library_softmax():
    # Q block i is constant (a_i, 0, ..), K block j constant (b_j, 0, ..): Sbar_ij = a_i b_j / sqrt(d)
    d = 4
    a = np.array([0.5, -1.0, 2.0]); b = np.array([1.0, 0.0, -2.0, 3.0, 0.25, -0.75])
    q = np.zeros((3 * 128, d)); k = np.zeros((6 * 64, d))
    q[:, 0] = np.repeat(a, 128); k[:, 0] = np.repeat(b, 64)
    k[:, 1] = 7.0                                 # orthogonal to q: must not matter
    # zero-mean offsets inside each block: +-0.5 on the two halves of a 128-token query block and of a 64-token
    # key block.  They cancel only if Q is averaged over 128 tokens and K over 64.
    q[:, 0] += np.tile(np.repeat([0.5, -0.5], 64), 3)
    k[:, 0] += np.tile(np.repeat([0.5, -0.5], 32), 6)
    n = 384
    pbar = orc.pooled_map(q[:n], k[:n])
    expect = scipy_softmax(np.outer(a, b) / math.sqrt(d), axis=1)
    np.testing.assert_allclose(pbar, expect, rtol=1e-14)
    # logits far beyond exp's range: the row softmax still matches the library's
    big = np.array([[1000.0, 999.0, -1000.0], [-800.0, -801.0, -802.0]])
    np.testing.assert_allclose(orc.softmax_rows(big), scipy_softmax(big, axis=1), rtol=1e-14)
    # transposing the roles of Q and K would give a 6x3 map / different numbers
    assert pbar.shape == (3, 6)


# ------------------------------------------------------------------ attention forward
def _rand_problem(n, d, seed, t_keep=0.4):
    rng = np.random.default_rng(seed)
    q, k, v, do = (rng.normal(size=(n, d)) for _ in range(4))
    t_m, t_n = orc.num_blocks(n, 128), orc.num_blocks(n, 64)
    m = (rng.random((t_m, t_n)) < t_keep).astype(np.uint8)
    m[np.arange(t_m), rng.integers(0, t_n, t_m)] = 1
    return q, k, v, do, m


def test_full_mask_equals_library_dense_attention():
    q, k, v, _, m = _rand_problem(300, 16, 3)
    m[:] = 1
    o, lse, p = orc.attention_definition(q, k, v, m)
    tq, tk, tv = (torch.from_numpy(x)[None, None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, 0].numpy()
    np.testing.assert_allclose(o, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-14)
    ref_lse = torch.logsumexp(tq[0, 0] @ tk[0, 0].T / math.sqrt(16), dim=1).numpy()
    np.testing.assert_allclose(lse, ref_lse, rtol=1e-13)


@pytest.mark.parametrize("n,d,seed", [(300, 16, 4), (512, 32, 5), (700, 8, 6)])
def test_masked_attention_three_forms_and_library_masked_sdpa(n, d, seed):
    q, k, v, _, m = _rand_problem(n, d, seed)
    o1, lse1, p = orc.attention_definition(q, k, v, m)
    o2, lse2 = orc.attention_gather(q, k, v, m)
    o3, lse3 = orc.attention_tile_merge(q, k, v, m)
    np.testing.assert_allclose(o2, o1, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(o3, o1, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(lse2, lse1, rtol=1e-13)
    np.testing.assert_allclose(lse3, lse1, rtol=1e-13)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-14)
    keep = torch.from_numpy(orc.expand_mask(m, n))
    tq, tk, tv = (torch.from_numpy(x)[None, None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=keep[None, None])[0, 0].numpy()
    np.testing.assert_allclose(o1, ref, rtol=1e-11, atol=1e-13)
    # masked weights are exactly zero, kept tiles are not
    assert (p[~keep.numpy()] == 0).all() and (p[keep.numpy()] > 0).all()


def test_error_decomposition_identity_on_attention_outputs():
    """o - o_s = (p(.)(1-m)) V + (1 - 1/tau) (p(.)m) V with o, o_s taken from the attention routines."""
    rng = np.random.default_rng(7)
    n, d = 12, 5
    q, k, v = (rng.normal(size=(n, d)) for _ in range(3))
    m = (rng.random((n, n)) < 0.5).astype(np.uint8); m[np.arange(n), np.arange(n)] = 1
    full, _, p_full = orc.attention_definition(q, k, v, np.ones((n, n), np.uint8), bq=1, bkv=1)
    sparse, _, p_sparse = orc.attention_definition(q, k, v, m, bq=1, bkv=1)
    for r in range(n):
        tau, o, o_s, dropped, renorm = orc.error_terms(p_full[r], m[r], v)
        np.testing.assert_allclose(o, full[r], atol=1e-14)
        np.testing.assert_allclose(o_s, sparse[r], atol=1e-13)
        np.testing.assert_allclose(full[r] - sparse[r], dropped + renorm, atol=1e-13)
        np.testing.assert_allclose(p_sparse[r], p_full[r] * m[r] / tau, atol=1e-14)


def test_single_block_with_identical_keys_gives_mean_of_values():
    n, d = 256, 8
    rng = np.random.default_rng(8)
    q = rng.normal(size=(n, d)); v = rng.normal(size=(n, d))
    k = rng.normal(size=(n, d)); k[64:128] = k[64]          # block 1: identical keys
    m = np.zeros((2, 4), np.uint8); m[:, 1] = 1
    for f in (orc.attention_gather, orc.attention_tile_merge):
        o, lse = f(q, k, v, m)
        np.testing.assert_allclose(o, np.tile(v[64:128].mean(axis=0), (n, 1)), atol=1e-13)
        np.testing.assert_allclose(lse, q @ k[64] / math.sqrt(d) + math.log(64), rtol=1e-12, atol=1e-12)


def test_short_last_blocks():
    # N = 300: q blocks of 128,128,44 rows; kv blocks 64,64,64,64,44
    q, k, v, _, m = _rand_problem(300, 8, 9)
    assert m.shape == (3, 5)
    m[:, 4] = 1
    o1, _, p = orc.attention_definition(q, k, v, m)
    o2, _ = orc.attention_gather(q, k, v, m)
    assert o1.shape == (300, 8) and p.shape == (300, 300)
    np.testing.assert_allclose(o2, o1, rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------------ gradients
def _loss(q, k, v, m, do):
    o, _, _ = orc.attention_definition(q, k, v, m)
    return float((o * do).sum())


def test_gradients_match_central_finite_differences():
    q, k, v, do, m = _rand_problem(200, 6, 10, t_keep=0.5)
    dq, dk, dv = orc.attention_bwd_definition(q, k, v, m, do)
    rng = np.random.default_rng(11)
    eps = 1e-5
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        for _ in range(12):
            r, c = rng.integers(0, x.shape[0]), rng.integers(0, x.shape[1])
            old = x[r, c]
            x[r, c] = old + eps; up = _loss(q, k, v, m, do)
            x[r, c] = old - eps; dn = _loss(q, k, v, m, do)
            x[r, c] = old
            fd = (up - dn) / (2 * eps)
            assert fd == pytest.approx(g[r, c], rel=1e-6, abs=1e-8), (name, r, c)
    # directional derivative over everything at once
    dirs = [rng.normal(size=x.shape) for x in (q, k, v)]
    up = _loss(q + eps * dirs[0], k + eps * dirs[1], v + eps * dirs[2], m, do)
    dn = _loss(q - eps * dirs[0], k - eps * dirs[1], v - eps * dirs[2], m, do)
    ana = (dq * dirs[0]).sum() + (dk * dirs[1]).sum() + (dv * dirs[2]).sum()
    assert (up - dn) / (2 * eps) == pytest.approx(ana, rel=1e-7)


@pytest.mark.parametrize("n,d,seed", [(300, 16, 12), (520, 8, 13)])
def test_gradients_match_library_autograd_and_gather_form(n, d, seed):
    q, k, v, do, m = _rand_problem(n, d, seed)
    dq, dk, dv = orc.attention_bwd_definition(q, k, v, m, do)
    tq, tk, tv = (torch.from_numpy(x).clone().requires_grad_(True) for x in (q, k, v))
    keep = torch.from_numpy(orc.expand_mask(m, n))
    s = (tq @ tk.T) / math.sqrt(d)
    o = torch.softmax(s.masked_fill(~keep, float("-inf")), dim=1) @ tv
    o.backward(torch.from_numpy(do))
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-12)
    gq, gk, gv, go, glse = orc.attention_bwd_gather(q, k, v, m, do)
    np.testing.assert_allclose(gq, dq, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(gk, dk, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(gv, dv, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(go, o.detach().numpy(), rtol=1e-10, atol=1e-12)


def test_gradient_closed_forms():
    n, d = 256, 4
    rng = np.random.default_rng(14)
    k, v, do = (rng.normal(size=(n, d)) for _ in range(3))
    m = np.ones((2, 4), np.uint8)
    # Q = 0 and the full mask: P is uniform, so dV_c = mean_r dO_r for every c, and dK = 0
    dq, dk, dv = orc.attention_bwd_definition(np.zeros((n, d)), k, v, m, do)
    np.testing.assert_allclose(dv, np.tile(do.mean(axis=0), (n, 1)), atol=1e-14)
    np.testing.assert_allclose(dk, 0.0, atol=1e-14)
    # keys of a never-selected block receive exactly zero gradient
    m2 = np.ones((2, 4), np.uint8); m2[:, 2] = 0
    q = rng.normal(size=(n, d))
    dq, dk, dv = orc.attention_bwd_definition(q, k, v, m2, do)
    assert (dk[128:192] == 0).all() and (dv[128:192] == 0).all()
    # softmax is invariant to adding a constant to a row of logits, so the rows of dS sum to zero
    o, _, p = orc.attention_definition(q, k, v, m2)
    dp = do @ v.T
    ds = p * (dp - (do * o).sum(axis=1, keepdims=True))
    np.testing.assert_allclose(ds.sum(axis=1), 0.0, atol=1e-12)
    np.testing.assert_allclose(dq, ds @ k / math.sqrt(d), atol=1e-13)


def test_batched_wrappers_are_per_head():
    rng = np.random.default_rng(15)
    q, k, v, do = (rng.normal(size=(2, 2, 256, 8)) for _ in range(4))
    mask, pbar = orc.block_mask_bh(q, k, 2, 0.5)
    assert mask.shape == (2, 2, 2, 4)
    for b in range(2):
        for h in range(2):
            m1, p1 = orc.block_mask(q[b, h], k[b, h], 2, 0.5)
            assert np.array_equal(mask[b, h], m1)
            np.testing.assert_array_equal(pbar[b, h], p1)
    o, lse = orc.attention_bh(q, k, v, mask)
    dq, dk, dv, o2, lse2 = orc.attention_bwd_bh(q, k, v, mask, do)
    np.testing.assert_allclose(o, o2, atol=1e-14)
    e_o, e_lse, _ = orc.attention_definition(q[1, 0], k[1, 0], v[1, 0], mask[1, 0])
    np.testing.assert_allclose(o2[1, 0], e_o, atol=1e-13)
    np.testing.assert_allclose(lse2[1, 0], e_lse, atol=1e-13)
    np.testing.assert_allclose(lse[1, 0], e_lse, atol=1e-13)
    e_dq, e_dk, e_dv = orc.attention_bwd_definition(q[0, 1], k[0, 1], v[0, 1], mask[0, 1], do[0, 1])
    np.testing.assert_allclose(dq[0, 1], e_dq, atol=1e-12)
    np.testing.assert_allclose(dk[0, 1], e_dk, atol=1e-12)
    np.testing.assert_allclose(dv[0, 1], e_dv, atol=1e-12)


def test_q_blocks_subset_matches_full_evaluation():
    q, k, v, do, m = _rand_problem(700, 8, 21)
    full = orc.attention_bwd_gather(q, k, v, m, do)
    sub = orc.attention_bwd_gather(q, k, v, m, do, q_blocks=[1, 4])
    for r0, r1 in ((128, 256), (512, 640)):
        for a, b in zip((full[0], full[3], full[4]), (sub[0], sub[3], sub[4])):     # dQ, O, LSE rows
            np.testing.assert_array_equal(a[r0:r1], b[r0:r1])
    assert (sub[3][:128] == 0).all()
    # a key block's gradient is complete once every query block of its column is visited
    j = 3
    rows = [int(i) for i in np.flatnonzero(m[:, j])]
    part = orc.attention_bwd_gather(q, k, v, m, do, q_blocks=rows)
    np.testing.assert_allclose(part[1][j * 64:(j + 1) * 64], full[1][j * 64:(j + 1) * 64], atol=1e-13)
    np.testing.assert_allclose(part[2][j * 64:(j + 1) * 64], full[2][j * 64:(j + 1) * 64], atol=1e-13)
    o_sub, lse_sub = orc.attention_gather(q, k, v, m, q_blocks=[2])
    o_all, lse_all = orc.attention_gather(q, k, v, m)
    np.testing.assert_array_equal(o_sub[256:384], o_all[256:384])


# ------------------------------------------------------------------ Sec. 3.1 summed over a head
def test_error_sums_identities():
    """tau of a row equals exp(LSE_sparse - LSE_full); the two parts add up to the error row by row, so the
    L1 norm of the total is at most the sum of the L1 norms of the parts; a full mask has no error."""
    rng = np.random.default_rng(11)
    n, d = 300, 16
    q, k, v = rng.standard_normal((3, n, d))
    mbar, _ = orc.block_mask(q, k, 1, 0.5)
    tot, ref, drop, ren, tau_sum = orc.error_sums(q, k, v, mbar)
    _, lse_s = orc.attention_gather(q, k, v, mbar)
    _, lse_f = orc.attention_gather(q, k, v, np.ones_like(mbar))
    assert abs(np.exp(lse_s - lse_f).sum() - tau_sum) < 1e-9
    assert 0 < tot <= drop + ren + 1e-12 and ref > 0
    # against the outputs themselves: o - o_s from the two attention calls
    o_s, _ = orc.attention_gather(q, k, v, mbar)
    o_f = orc.attention_definition(q, k, v, np.ones_like(mbar))[0]
    assert abs(np.abs(o_f - o_s).sum() - tot) < 1e-9 * max(1.0, tot)
    assert abs(np.abs(o_f).sum() - ref) < 1e-9 * ref
    # which part is which: every row keeps the same key blocks, V is 1 on kept tokens and 0 on dropped ones.
    # Then the dropped weights carry nothing (dropped error 0) and the kept ones, rescaled by 1/tau, give
    # o_s = 1 against o = tau: the renormalisation error is (tau - 1) in each of the d channels.
    same = np.zeros_like(mbar); same[:, [0, 3]] = 1
    vk = np.zeros((n, d)); vk[0:64] = 1.0; vk[192:256] = 1.0
    tot2, ref2, drop2, ren2, tau2 = orc.error_sums(q, k, vk, same)
    assert drop2 < 1e-12 and abs(ren2 - d * (n - tau2)) < 1e-9 and abs(tot2 - ren2) < 1e-9
    assert abs(ref2 - d * tau2) < 1e-9
    full = orc.error_sums(q, k, v, np.ones_like(mbar))
    assert full[0] < 1e-12 and full[2] < 1e-12 and full[3] < 1e-12 and abs(full[4] - n) < 1e-9


# ------------------------------------------------------------------ velocity distillation loss
def test_vd_loss_closed_forms_and_library_gradient():
    rng = np.random.default_rng(31)
    u_f = rng.normal(size=(3, 50, 8))
    # equal predictions: no loss, no gradient; a constant offset c over n elements: weight * n * c^2
    loss, grad = orc.vd_loss(u_f, u_f, 0.25)
    assert loss == 0.0 and not grad.any()
    loss, grad = orc.vd_loss(u_f + 0.5, u_f, 1.0 / 3)                 # three samples of 400 elements
    assert abs(loss - 400 * 0.25) < 1e-10
    np.testing.assert_allclose(grad, 2 * 0.5 / 3, rtol=1e-12)
    # the sign: the gradient points from the teacher to the student
    u_s = u_f.copy(); u_s[1, 7, 2] += 2.0
    loss, grad = orc.vd_loss(u_s, u_f, 1.0)
    assert abs(loss - 4.0) < 1e-12 and abs(grad[1, 7, 2] - 4.0) < 1e-12 and np.count_nonzero(grad) == 1
    # against the library: mean-squared error and autograd in fp64
    u_s = rng.normal(size=u_f.shape)
    ts = torch.tensor(u_s, dtype=torch.float64, requires_grad=True)
    tl = torch.nn.functional.mse_loss(ts, torch.tensor(u_f, dtype=torch.float64))
    tl.backward()
    loss, grad = orc.vd_loss(u_s, u_f, 1.0 / u_s.size)
    assert abs(loss - tl.item()) < 1e-14
    np.testing.assert_allclose(grad, ts.grad.numpy(), rtol=1e-13, atol=1e-18)


def test_parts_of_a_row_merge_to_the_whole_row():
    """The identity behind splitting a long row over several workgroups: evaluate the attention of a query block
    over disjoint subsets of its selected key blocks separately (each with its own softmax), then combine the
    partial outputs with weights exp(LSE_part - LSE) -- Alg. 1 step 18's division by the total row sum is what makes
    this equal to one softmax over all selected keys.  Checked against the definition, with uneven parts."""
    q, k, v, _, m = _rand_problem(700, 16, 11)
    m[:] = 0
    rng = np.random.default_rng(12)
    for i in range(m.shape[0]):
        m[i, rng.choice(m.shape[1], size=7, replace=False)] = 1
    o_ref, lse_ref, _ = orc.attention_definition(q, k, v, m)
    for cuts in ((3,), (1, 2), (2, 5, 6)):
        outs, lses = [], []
        for i in range(m.shape[0]):
            sel = np.flatnonzero(m[i])
            bounds = (0,) + cuts + (sel.size,)
            o_parts, lse_parts = [], []
            for a, b in zip(bounds[:-1], bounds[1:]):
                part = np.zeros_like(m); part[i, sel[a:b]] = 1
                o_p, lse_p = orc.attention_gather(q, k, v, part, q_blocks=[i])
                r0, r1 = i * 128, min(700, (i + 1) * 128)
                o_parts.append(o_p[r0:r1]); lse_parts.append(lse_p[r0:r1])
            stack = np.stack(lse_parts, axis=1)
            top = stack.max(axis=1, keepdims=True)
            lse = (top + np.log(np.exp(stack - top).sum(axis=1, keepdims=True)))[:, 0]
            outs.append(sum(np.exp(lp - lse)[:, None] * op for lp, op in zip(lse_parts, o_parts)))
            lses.append(lse)
        np.testing.assert_allclose(np.concatenate(outs), o_ref, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(np.concatenate(lses), lse_ref, rtol=1e-13)
