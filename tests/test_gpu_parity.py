"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by
element, on seeded inputs small enough for the oracle but spanning several tiles and
ragged tails."""
import dataclasses
import math

import numpy as np
import pytest
import torch

import paper_2602_13515_amd as spa2
from oracle import spa2_oracle as orc
from paper_2602_13515_amd import workloads as wl

from gpu_util import (LOWRANK_MAX_ABS, assert_close, check_pattern_consistency, dev, f64, gpu_bwd, gpu_fwd, gpu_mask,
                      mask_protocol, pattern_from_mask)

pytestmark = pytest.mark.gpu


def _small(name, N, d, kind="gaussian", H=2, B=1, k=0.25, p=0.9):
    return wl.Workload(name, B, H, N, d, k, p, kind, True)


def _random_mask(B, H, N, keep, seed):
    rng = np.random.default_rng(seed)
    Tm, Tn = -(-N // 128), -(-N // 64)
    m = (rng.random((B, H, Tm, Tn)) < keep).astype(np.uint8)
    for b in range(B):
        for h in range(H):
            m[b, h, np.arange(Tm), rng.integers(0, Tn, Tm)] = 1
    return m


FWD_CASES = [
    ("tiny-d64", wl.TINY, 0.3),
    ("ragged-d128", _small("ragged128", 1000, 128), 0.4),       # last q block 104 rows, last kv block 40 keys
    ("ragged-d64", _small("ragged64", 1110, 64), 0.5),          # 86 / 22
    ("one-block", _small("one", 64, 128, H=1), 1.0),
    ("short", _small("short", 17, 64, H=1), 1.0),
]


@pytest.mark.parametrize("name,w,keep", FWD_CASES, ids=[c[0] for c in FWD_CASES])
def test_fwd_bwd_on_given_pattern(name, w, keep):
    print(f"case {name}: B={w.B} H={w.H} N={w.N} d={w.d}", flush=True)
    q, k, v, do = wl.make_inputs(w, seed=1)
    mask = _random_mask(w.B, w.H, w.N, keep, seed=2)
    qd, kd, vd, dod = (t.to(dev()) for t in (q, k, v, do))
    pat = pattern_from_mask(mask, dev())
    o, lse = gpu_fwd(qd, kd, vd, pat)
    dq, dk, dv = gpu_bwd(qd, kd, vd, o, dod, lse, pat)
    r_dq, r_dk, r_dv, r_o, r_lse = orc.attention_bwd_bh(f64(q), f64(k), f64(v), mask, f64(do))
    print("O", assert_close("O", f64(o), r_o))
    assert np.abs(f64(lse) - r_lse).max() <= 2e-3
    # gradients: the GPU consumes its own bf16 O and fp32 LSE, as a training step would
    print("dQ", assert_close("dQ", f64(dq), r_dq))
    print("dK", assert_close("dK", f64(dk), r_dk))
    print("dV", assert_close("dV", f64(dv), r_dv))


def test_block_edges_sweep():
    """Token counts on both sides of every block edge (64 and 128 tokens) and a few seeded odd ones, both head
    dimensions, the masker's own pattern: mask protocol, then O, LSE and the three gradients element by element."""
    rng = np.random.default_rng(77)
    counts = [63, 65, 127, 129, 191, 193, 255, 257, 1279, 1281] + [int(x) for x in rng.integers(300, 3000, size=4)]
    for n_i, N in enumerate(counts):
        d = 128 if n_i % 2 == 0 else 64
        w = _small(f"edge{N}", N, d, kind="gaussian" if n_i % 3 else "lowrank", H=2, k=0.3, p=0.6)
        print(f"case N={N} d={d} kind={w.kind}", flush=True)
        q, k, v, do = wl.make_inputs(w, seed=100 + N)
        qd, kd, vd, dod = (t.to(dev()) for t in (q, k, v, do))
        k_cnt = spa2.spa2_topk_blocks(w.k_frac, w.Tn)
        pat, pbar = gpu_mask(qd, kd, k_cnt, w.top_p)
        mask = check_pattern_consistency(pat)
        for h in range(w.H):
            rep = mask_protocol(mask[0, h], pbar[0, h].cpu().numpy(), orc.pooled_map(f64(q)[0, h], f64(k)[0, h]),
                                k_cnt, w.top_p)
            assert rep["stage1_max_rel"] <= 1e-5 and rep["stage2_unexplained"] == 0 and rep["stage3_unexplained"] == 0, (N, h, rep)
        o, lse = gpu_fwd(qd, kd, vd, pat)
        dq, dk, dv = gpu_bwd(qd, kd, vd, o, dod, lse, pat)
        r_dq, r_dk, r_dv, r_o, r_lse = orc.attention_bwd_bh(f64(q), f64(k), f64(v), mask, f64(do))
        assert_close(f"O N={N}", f64(o), r_o)
        assert np.abs(f64(lse) - r_lse).max() <= 2e-3
        # low-rank inputs: dS, rounded to bf16, meets keys and queries of magnitude 8-10 in dQ = dS K and dK = dS^T Q;
        # the rounding alone, applied to an exact computation on the CPU, moves single elements by 3-4e-2
        big = LOWRANK_MAX_ABS if w.kind == "lowrank" else 2e-2
        assert_close(f"dQ N={N}", f64(dq), r_dq, max_abs=big)
        assert_close(f"dK N={N}", f64(dk), r_dk, max_abs=big)
        assert_close(f"dV N={N}", f64(dv), r_dv)


def test_full_pattern_is_dense_attention():
    w = _small("dense", 700, 128, H=2)
    q, k, v, do = wl.make_inputs(w, seed=3)
    qd, kd, vd, dod = (t.to(dev()) for t in (q, k, v, do))
    pat = spa2.alloc_pattern(w.B, w.H, w.N, dev())
    spa2.spa2_pattern_full(qd, pat)
    torch.cuda.synchronize()
    mask = check_pattern_consistency(pat)
    assert mask.all()
    o, lse = gpu_fwd(qd, kd, vd, pat)
    dq, dk, dv = gpu_bwd(qd, kd, vd, o, dod, lse, pat)
    for h in range(w.H):
        r_o, r_lse, _ = orc.attention_definition(f64(q)[0, h], f64(k)[0, h], f64(v)[0, h], mask[0, h])
        r_dq, r_dk, r_dv = orc.attention_bwd_definition(f64(q)[0, h], f64(k)[0, h], f64(v)[0, h], mask[0, h], f64(do)[0, h])
        assert_close("O", f64(o)[0, h], r_o)
        assert_close("dQ", f64(dq)[0, h], r_dq)
        assert_close("dK", f64(dk)[0, h], r_dk)
        assert_close("dV", f64(dv)[0, h], r_dv)
        assert np.abs(f64(lse)[0, h] - r_lse).max() <= 2e-3


MASK_CASES = [
    ("tiny", wl.TINY, 0.25, 0.9),
    ("ragged-lowrank", _small("rl", 5000, 128, kind="lowrank", H=3), 0.05, 0.8),
    ("ragged-lowrank-topp-only", _small("rl2", 5000, 128, kind="lowrank", H=2), 0.0, 0.6),
    ("lowrank-topk-only", _small("rl3", 4096, 64, kind="lowrank", H=2), 0.1, 0.0),
    ("stress-small", _small("st", 8192, 128, kind="stress", H=2, B=2), 0.05, 0.8),
    ("wide-row", _small("wide", 20000, 64, kind="lowrank", H=1), 0.03, 0.5),     # Tn = 313 -> 512-wide sort
    ("very-short", _small("vs", 100, 64, H=1), 0.5, 0.5),
    ("longest-row", _small("max", 64 * 8192 - 30, 64, kind="lowrank", H=1), 0.01, 0.3),   # Tn = 8192, the widest row
    ("everything", _small("all", 3000, 128, H=2), 1.0, 1.0),                              # k = 100 %: full mask
    # layers with many (batch, head) pairs and rows of at most 1536 blocks take the sixteen-rows-per-workgroup
    # selection kernel (scores on the fp64 matrix cores), like the 75,600-token layer of test_gpu_fullsize.py:
    # both head dimensions, ragged last row group and last column tile, hybrid / Top-p-only / Top-k-only
    ("many-heads-d64", _small("mh64", 16384 - 37, 64, kind="lowrank", H=16, B=8), 0.1, 0.7),        # T_n = 256
    ("many-heads-d64-topp-only", _small("mh64p", 16384 - 37, 64, kind="lowrank", H=16, B=8), 0.0, 0.6),
    ("many-heads-d128", _small("mh128", 44800 - 5 - 64 * 3, 128, kind="stress", H=12, B=4), 0.05, 0.8),   # T_m = 349, T_n = 697
    ("many-heads-d128-topk-only", _small("mh128k", 30000, 128, kind="lowrank", H=10, B=7), 0.08, 0.0),    # T_n = 469
    ("many-heads-1024-wide", _small("mh1024", 60000 + 11, 64, kind="lowrank", H=12, B=3), 0.04, 0.85),    # T_n = 938
    ("many-heads-1536-wide", _small("mh1536", 90000 - 70, 128, kind="stress", H=8, B=3), 0.03, 0.9),      # T_n = 1406
]


@pytest.mark.parametrize("name,w,kf,p", MASK_CASES, ids=[c[0] for c in MASK_CASES])
def test_mask_protocol(name, w, kf, p):
    print(f"case {name}: B={w.B} H={w.H} N={w.N} d={w.d} k={kf} p={p}", flush=True)
    q, k, _, _ = wl.make_inputs(w, seed=4, need_do=False)
    k_cnt = spa2.spa2_topk_blocks(kf, w.Tn)
    assert k_cnt == orc.topk_blocks(kf, w.Tn)
    pat, pbar = gpu_mask(q.to(dev()), k.to(dev()), k_cnt, p)
    mask = check_pattern_consistency(pat)
    pbar = pbar.cpu().numpy()
    assert np.isfinite(pbar).all()
    tot = dict(stage2_near_cut=0, stage3_hamming=0, stage3_near_cut=0, stage3_ulp_swap=0)
    for b in range(w.B):
        for h in range(w.H):
            ref_pbar = orc.pooled_map(f64(q)[b, h], f64(k)[b, h])
            r = mask_protocol(mask[b, h], pbar[b, h], ref_pbar, k_cnt, p)
            assert r["stage1_max_rel"] <= 1e-5, r
            assert r["stage2_unexplained"] == 0, r
            assert r["stage3_unexplained"] == 0, r
            for key in tot:
                tot[key] += r[key]
            # invariants of the rule on the GPU mask itself
            assert (mask[b, h].sum(1) >= max(1, k_cnt)).all()
            sel_mass = (ref_pbar * mask[b, h]).sum(1)
            assert ((sel_mass >= np.float32(p) - 1e-5) | mask[b, h].all(1)).all()
    print("flip counts:", tot, "density:", mask.mean())


def test_end_to_end_tiny_mask_then_attention():
    """The benchmark's small configuration, whole path: mask -> fwd -> bwd."""
    w = wl.TINY
    q, k, v, do = wl.make_inputs(w, seed=0)
    qd, kd, vd, dod = (t.to(dev()) for t in (q, k, v, do))
    k_cnt = spa2.spa2_topk_blocks(w.k_frac, w.Tn)
    pat, _ = gpu_mask(qd, kd, k_cnt, w.top_p)
    mask = check_pattern_consistency(pat)
    o, lse = gpu_fwd(qd, kd, vd, pat)
    dq, dk, dv = gpu_bwd(qd, kd, vd, o, dod, lse, pat)
    # attention parity uses the GPU's mask on both sides, so a boundary flip cannot leak in
    r_dq, r_dk, r_dv, r_o, r_lse = orc.attention_bwd_bh(f64(q), f64(k), f64(v), mask, f64(do))
    assert_close("O", f64(o), r_o)
    assert_close("dQ", f64(dq), r_dq)
    assert_close("dK", f64(dk), r_dk)
    assert_close("dV", f64(dv), r_dv)
    ref_mask, _ = orc.block_mask_bh(f64(q), f64(k), k_cnt, float(np.float32(w.top_p)))
    print("hamming distance to the fp64 mask:", int((ref_mask != mask).sum()))


def test_strided_layout_bnhd():
    """[B, N, H, d] storage viewed as [B, H, N, d]: same results as the contiguous layout."""
    w = _small("strided", 600, 128, H=3)
    q, k, v, do = wl.make_inputs(w, seed=5)
    mask = _random_mask(w.B, w.H, w.N, 0.5, seed=6)
    pat = pattern_from_mask(mask, dev())

    def bnhd(t):
        return t.to(dev()).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)

    qs, ks, vs, dos = bnhd(q), bnhd(k), bnhd(v), bnhd(do)
    assert not qs.is_contiguous()
    o = torch.empty_like(qs); lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=dev())
    spa2.spa2_fwd(qs, ks, vs, pat, 1 / math.sqrt(w.d), o, lse)
    dq, dk, dv = torch.empty_like(qs), torch.empty_like(qs), torch.empty_like(qs)
    ws = torch.empty(spa2.spa2_bwd_workspace_bytes(qs), dtype=torch.uint8, device=dev())
    spa2.spa2_bwd(qs, ks, vs, o, dos, lse, pat, 1 / math.sqrt(w.d), dq, dk, dv, ws)
    pat2, pbar2 = gpu_mask(qs, ks, 3, 0.5)
    pat3, pbar3 = gpu_mask(q.to(dev()), k.to(dev()), 3, 0.5)
    torch.cuda.synchronize()
    assert torch.equal(pat2.mask, pat3.mask) and torch.equal(pbar2, pbar3)
    r_dq, r_dk, r_dv, r_o, _ = orc.attention_bwd_bh(f64(q), f64(k), f64(v), mask, f64(do))
    assert_close("O", f64(o), r_o)
    assert_close("dQ", f64(dq), r_dq)
    assert_close("dK", f64(dk), r_dk)
    assert_close("dV", f64(dv), r_dv)


def test_output_residual_recovers_fp32_output():
    """o + o_res carries the forward result to about 16 mantissa bits, and the backward pass that is
    given o_res computes D = rowsum(dO * O) from it."""
    w = _small("res", 2000, 128, kind="lowrank", H=2)
    q, k, v, do = wl.make_inputs(w, seed=10)
    qd, kd, vd, dod = (t.to(dev()) for t in (q, k, v, do))
    pat, _ = gpu_mask(qd, kd, 4, 0.7)
    mask = pat.mask.cpu().numpy()
    o, lse, o_res = gpu_fwd(qd, kd, vd, pat, residual=True)
    o_plain, lse_plain = gpu_fwd(qd, kd, vd, pat)
    assert torch.equal(o, o_plain) and torch.equal(lse, lse_plain)
    r_dq, r_dk, r_dv, r_o, _ = orc.attention_bwd_bh(f64(q), f64(k), f64(v), mask, f64(do))
    err_hi = np.abs(f64(o) - r_o).max()
    err_sum = np.abs(f64(o) + f64(o_res) - r_o).max()
    print("max |o - O|", err_hi, " max |o + o_res - O|", err_sum)
    # the fp32 accumulator itself carries the error of the bf16-rounded P (2^-9 per term), so the sum is
    # not exact; it is several times closer than the rounded output alone
    assert err_sum < err_hi / 2
    dq1, dk1, dv1 = gpu_bwd(qd, kd, vd, o, dod, lse, pat)
    dq2, dk2, dv2 = gpu_bwd(qd, kd, vd, o, dod, lse, pat, o_res=o_res)
    e1 = np.abs(f64(dq1) - r_dq).max(); e2 = np.abs(f64(dq2) - r_dq).max()
    print("dQ max-abs error without / with residual:", e1, e2)
    assert e2 <= e1 * 1.05
    # low-rank workload, |K| ~ 10: the bf16 rounding of dS alone reaches 3e-2 on single elements of dQ
    assert_close("dQ", f64(dq2), r_dq, max_abs=LOWRANK_MAX_ABS); assert_close("dK", f64(dk2), r_dk); assert_close("dV", f64(dv2), r_dv)
    assert torch.equal(dv1, dv2)           # dV does not depend on D


def test_launch_orders_do_not_change_results():
    """row_order / col_order only permute which workgroup does which block."""
    w = _small("ord", 3000, 128, kind="lowrank", H=2)
    q, k, v, do = (t.to(dev()) for t in wl.make_inputs(w, seed=9))
    pat, _ = gpu_mask(q, k, 4, 0.7)
    assert pat.col_order is not None
    o1, lse1 = gpu_fwd(q, k, v, pat)
    g1 = gpu_bwd(q, k, v, o1, do, lse1, pat)
    plain = spa2.Pattern(pat.mask, pat.row_cnt, pat.row_idx, pat.col_cnt, pat.col_idx, None, None)
    o2, lse2 = gpu_fwd(q, k, v, plain)
    g2 = gpu_bwd(q, k, v, o2, do, lse2, plain)
    gen = torch.Generator().manual_seed(0)
    perm_r = torch.stack([torch.randperm(w.Tm, generator=gen) for _ in range(w.B * w.H)]).view(w.B, w.H, w.Tm)
    perm_c = torch.stack([torch.randperm(w.Tn, generator=gen) for _ in range(w.B * w.H)]).view(w.B, w.H, w.Tn)
    shuffled = spa2.Pattern(pat.mask, pat.row_cnt, pat.row_idx, pat.col_cnt, pat.col_idx,
                            perm_r.int().to(dev()), perm_c.int().to(dev()))
    o3, lse3 = gpu_fwd(q, k, v, shuffled)
    g3 = gpu_bwd(q, k, v, o3, do, lse3, shuffled)
    for a, b, c in zip((o1, lse1, *g1), (o2, lse2, *g2), (o3, lse3, *g3)):
        assert torch.equal(a, b) and torch.equal(a, c)


def test_kernels_are_deterministic():
    w = _small("det", 1500, 128, kind="lowrank", H=2)
    q, k, v, do = (t.to(dev()) for t in wl.make_inputs(w, seed=7))
    outs = []
    for _ in range(2):
        pat, pbar = gpu_mask(q, k, 3, 0.7)
        o, lse = gpu_fwd(q, k, v, pat)
        dq, dk, dv = gpu_bwd(q, k, v, o, do, lse, pat)
        outs.append((pat.mask, pat.row_idx, pat.col_idx, pbar, o, lse, dq, dk, dv))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_sixteen_row_selection_is_deterministic():
    """The selection kernel of layers with many (batch, head) pairs builds its histograms with LDS atomics: counts
    and fixed-point masses are integers, so the pattern and the exported probabilities must be the same bits on
    every run."""
    w = _small("det16", 16384 - 37, 64, kind="lowrank", H=16, B=8)
    q, k, _, _ = wl.make_inputs(w, seed=5, need_do=False)
    qd, kd = q.to(dev()), k.to(dev())
    outs = []
    for _ in range(3):
        pat, pbar = gpu_mask(qd, kd, spa2.spa2_topk_blocks(0.1, w.Tn), 0.7)
        outs.append((pat.mask, pat.row_cnt, pat.row_idx, pat.col_cnt, pat.col_idx, pat.col_order, pbar))
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)


def test_error_codes_leave_outputs_untouched():
    w = _small("err", 256, 128, H=1)
    q, k, v, do = (t.to(dev()) for t in wl.make_inputs(w, seed=8))
    pat = spa2.alloc_pattern(1, 1, 256, dev())
    pat.mask.fill_(9)
    ws = torch.empty(spa2.spa2_mask_workspace_bytes(q), dtype=torch.uint8, device=dev())
    with pytest.raises(spa2.Spa2Error) as e:
        spa2.spa2_mask(q, k, 0, 0.0, 0.1, pat, None, ws)          # both rules off
    assert e.value.code == -5
    with pytest.raises(spa2.Spa2Error) as e:
        spa2.spa2_mask(q, k, 99, 0.5, 0.1, pat, None, ws)         # more blocks than the row has
    assert e.value.code == -5
    with pytest.raises(spa2.Spa2Error) as e:
        spa2.spa2_mask(q, k, 1, 0.5, 0.1, pat, None, ws[:16])     # workspace too small
    assert e.value.code == -6
    with pytest.raises(spa2.Spa2Error) as e:
        spa2.spa2_fwd(q[..., :32], k[..., :32], v[..., :32], pat, 0.1, q[..., :32], torch.empty(256, device=dev()))
    assert e.value.code == -3                                      # d = 32 unsupported
    torch.cuda.synchronize()
    assert (pat.mask == 9).all()


def test_whole_step_replays_from_a_hip_graph():
    """The library allocates nothing and never synchronises, so mask -> fwd -> bwd can be captured once and
    replayed; every replay (with eager work and synchronisations in between) must reproduce the eager result
    bit for bit."""
    w = _small("graph", 3000, 128, kind="lowrank", H=2, k=0.1, p=0.6)
    q, k, v, do = (t.to(dev()) for t in wl.make_inputs(w, seed=7))
    scale = 1.0 / math.sqrt(w.d)
    k_cnt = spa2.spa2_topk_blocks(w.k_frac, w.Tn)
    pat = spa2.alloc_pattern(w.B, w.H, w.N, dev())
    ws_m = torch.empty(spa2.spa2_mask_workspace_bytes(q), dtype=torch.uint8, device=dev())
    ws_b = torch.empty(spa2.spa2_bwd_workspace_bytes(q), dtype=torch.uint8, device=dev())
    ws_f = torch.empty(spa2.spa2_fwd_workspace_bytes(q), dtype=torch.uint8, device=dev())   # long rows are split
    o = torch.empty_like(q); o_res = torch.empty_like(q)
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=dev())
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)

    def step():
        spa2.spa2_mask(q, k, k_cnt, w.top_p, scale, pat, None, ws_m)
        spa2.spa2_fwd(q, k, v, pat, scale, o, lse, o_res, ws_f)
        spa2.spa2_bwd(q, k, v, o, do, lse, pat, scale, dq, dk, dv, ws_b, o_res)

    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in (pat.mask, o, lse, dq, dk, dv)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in (pat.mask, o, lse, dq, dk, dv, ws_f, ws_b):
            t.zero_()                            # eager work between the replays (plans and partial sums too)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, ref in zip(("mask", "O", "LSE", "dQ", "dK", "dV"), (pat.mask, o, lse, dq, dk, dv), eager):
            assert torch.equal(got, ref), (rep, name)


def test_long_rows_and_columns_are_split_and_merged():
    """A small layer whose longest rows and columns are several times the split length (Top-p-bound rows of the
    low-rank recipe, hot key blocks): with the workspaces, lists longer than S = max(16, tiles / 2048) are walked by
    several workgroups and merged in part order (Alg. 1 step 18: the final division makes the merge of (O, m, l)
    exact up to rounding).  Results must match the oracle to the same bars as the unsplit path, agree with the
    unsplit path to rounding, and be bit-identical from run to run."""
    w = _small("split", 9000, 128, kind="lowrank", H=2, k=0.05, p=0.8)          # T_m = 71, T_n = 141
    q, k, v, do = wl.make_inputs(w, seed=21)
    qd, kd, vd, dod = (t.to(dev()) for t in (q, k, v, do))
    k_cnt = spa2.spa2_topk_blocks(w.k_frac, w.Tn)
    pat, _ = gpu_mask(qd, kd, k_cnt, w.top_p, want_pbar=False)
    mask = check_pattern_consistency(pat)
    rc, cc = mask.sum(-1), mask.sum(-2)
    tiles = int(mask.sum())
    S_rows, S_cols = max(16, -(-tiles // 2048)), max(8, -(-tiles // 2048))
    print(f"tiles {tiles}; longest row {rc.max()} (split length {S_rows}), longest column {cc.max()} (split length {S_cols}); "
          f"rows split {(rc > S_rows).sum()}, columns split {(cc > S_cols).sum()}", flush=True)
    assert rc.max() > 3 * S_rows and cc.max() > 3 * S_cols, "the case must exercise several parts per list"
    runs = []
    for split in (True, True, False):
        o, lse, o_res = gpu_fwd(qd, kd, vd, pat, residual=True, split=split)
        dq, dk, dv = gpu_bwd(qd, kd, vd, o, dod, lse, pat, o_res=o_res, split=split)
        runs.append((o, lse, o_res, dq, dk, dv))
    for a, b in zip(runs[0], runs[1]):
        assert torch.equal(a, b), "split results must not depend on the order in which parts finish"
    r_dq, r_dk, r_dv, r_o, r_lse = orc.attention_bwd_bh(f64(q), f64(k), f64(v), mask, f64(do))
    for tag, (o, lse, o_res, dq, dk, dv) in (("split", runs[0]), ("whole", runs[2])):
        print(tag, "O", assert_close("O", f64(o), r_o))
        assert np.abs(f64(lse) - r_lse).max() <= 2e-3
        print(tag, "dQ", assert_close("dQ", f64(dq), r_dq, max_abs=LOWRANK_MAX_ABS))
        print(tag, "dK", assert_close("dK", f64(dk), r_dk, max_abs=LOWRANK_MAX_ABS))
        print(tag, "dV", assert_close("dV", f64(dv), r_dv))
    # The two paths differ by rounding only (another summation order; partial results stay fp32): stored bf16
    # values two spacings apart at most.  The forward outputs are compared directly (LSE: the row sum is taken over
    # P rounded against each part's own running maximum); the gradients are compared on the SAME forward outputs.
    o, lse, o_res = runs[0][:3]
    whole = gpu_bwd(qd, kd, vd, o, dod, lse, pat, o_res=o_res, split=False)
    pairs = [("O", runs[0][0], runs[2][0]), ("LSE", runs[0][1], runs[2][1])] + \
            [(n, a, b) for n, a, b in zip(("dQ", "dK", "dV"), runs[0][3:], whole)]
    for name, a, b in pairs:
        d = (a.float() - b.float()).abs()
        bound = 2.0 ** -6 * b.float().abs() + 1e-3 if name != "LSE" else torch.full_like(d, 1e-3)
        assert bool((d <= bound).all()), (name, float(d.max()))
