"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(stage entry points, column launch order): sampled outputs that the oracle can compute
one by one, plus properties that hold at any size."""
import math

import numpy as np
import pytest
import torch

import paper_2602_13515_amd as spa2
from oracle import spa2_oracle as orc
from paper_2602_13515_amd import workloads as wl

from gpu_util import MAX_ABS, MEAN_ABS, assert_close, dev, f64, mask_protocol

pytestmark = pytest.mark.gpu


def _run_path(w, q, k, v, do, k_frac=None, top_p=None, want_pbar=True):
    """mask -> fwd -> bwd exactly as bench.py sequences them."""
    k_frac = w.k_frac if k_frac is None else k_frac
    top_p = w.top_p if top_p is None else top_p
    scale = 1.0 / math.sqrt(w.d)
    k_cnt = spa2.spa2_topk_blocks(k_frac, w.Tn)
    pat = spa2.alloc_pattern(w.B, w.H, w.N, q.device)
    pbar = torch.empty((w.B, w.H, w.Tm, w.Tn), dtype=torch.float32, device=q.device) if want_pbar else None
    ws_m = torch.empty(spa2.spa2_mask_workspace_bytes(q), dtype=torch.uint8, device=q.device)
    ws_b = torch.empty(spa2.spa2_bwd_workspace_bytes(q), dtype=torch.uint8, device=q.device)
    o = torch.full_like(q, float("nan")); lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=q.device)
    o_res = torch.full_like(q, float("nan"))
    dq = torch.full_like(q, float("nan")); dk = torch.full_like(q, float("nan")); dv = torch.full_like(q, float("nan"))
    spa2.spa2_mask_pool(q, k, ws_m)
    spa2.spa2_mask_select(q, k_cnt, top_p, scale, pat, pbar, ws_m)
    spa2.spa2_mask_columns(q, pat)
    spa2.spa2_fwd(q, k, v, pat, scale, o, lse, o_res)
    spa2.spa2_bwd_delta(o, do, ws_b, o_res)
    spa2.spa2_bwd_dkdv(q, k, v, do, lse, pat, scale, dk, dv, ws_b)
    spa2.spa2_bwd_dq(q, k, v, do, lse, pat, scale, dq, ws_b)
    torch.cuda.synchronize()
    return k_cnt, pat, pbar, o, lse, dq, dk, dv


def _check_head_samples(w, b, h, q, k, v, do, pat, o, lse, dq, dk, dv, q_blocks, kv_blocks):
    """Oracle on one head, restricted to sampled query blocks (O, LSE, dQ rows) and to the query
    blocks that selected the sampled key blocks (dK, dV rows), using the GPU's own mask."""
    mask = pat.mask[b, h].cpu().numpy()
    qh, kh, vh, doh = (f64(t[b, h]) for t in (q, k, v, do))
    r_dq, _, _, r_o, r_lse = orc.attention_bwd_gather(qh, kh, vh, mask, doh, q_blocks=q_blocks)
    for i in q_blocks:
        r0, r1 = i * 128, min(w.N, (i + 1) * 128)
        assert_close(f"O[{b},{h}] block {i}", f64(o[b, h, r0:r1]), r_o[r0:r1])
        # dQ sums bf16-rounded dS (2^-9 relative) against keys of magnitude ~10 (the scale-2 low-rank part of
        # these workloads): single elements reach 3.3e-2 even in an otherwise exact numpy emulation of that
        # one rounding, which the GPU reproduces to 5e-3.  The plain 2e-2 bar is kept for O and dV and for
        # every small configuration; here dQ gets 5e-2 max-abs, the mean bar is unchanged.
        e = assert_close(f"dQ[{b},{h}] block {i}", f64(dq[b, h, r0:r1]), r_dq[r0:r1], max_abs=5e-2)
        print(f"  q block {i}: dQ max/mean err, elements above 2e-2: {e[0]:.4f} {e[1]:.5f} "
              f"{int((np.abs(f64(dq[b, h, r0:r1]) - r_dq[r0:r1]) > 2e-2).sum())}", flush=True)
        assert np.abs(f64(lse[b, h, r0:r1]) - r_lse[r0:r1]).max() <= 2e-3
    for j in kv_blocks:
        rows = [int(i) for i in np.flatnonzero(mask[:, j])]
        _, r_dk, r_dv, _, _ = orc.attention_bwd_gather(qh, kh, vh, mask, doh, q_blocks=rows)
        c0, c1 = j * 64, min(w.N, (j + 1) * 64)
        e = assert_close(f"dK[{b},{h}] block {j} ({len(rows)} query blocks)", f64(dk[b, h, c0:c1]), r_dk[c0:c1])
        assert_close(f"dV[{b},{h}] block {j}", f64(dv[b, h, c0:c1]), r_dv[c0:c1])
        print(f"  kv block {j}: {len(rows)} query blocks, dK max/mean err {e}", flush=True)


def _properties(w, pat, o, lse, dq, dk, dv, k_cnt):
    """Hold at any size: every output finite and fully written, pattern encodings agree in
    aggregate, every row keeps at least max(1, k_cnt) blocks."""
    for name, t in (("O", o), ("dQ", dq), ("dK", dk), ("dV", dv), ("LSE", lse)):
        assert torch.isfinite(t).all(), name
    m = pat.mask
    assert int(m.max()) <= 1
    assert torch.equal(pat.row_cnt.long(), m.sum(-1, dtype=torch.int64))
    assert torch.equal(pat.col_cnt.long(), m.sum(-2, dtype=torch.int64))
    assert int(pat.row_cnt.min()) >= max(1, k_cnt)
    srt = pat.col_order.sort(-1).values
    assert torch.equal(srt, torch.arange(w.Tn, device=srt.device, dtype=srt.dtype).expand_as(srt))
    # the index lists are ascending and consistent with the mask on a few random rows
    g = torch.Generator().manual_seed(0)
    for _ in range(16):
        b = int(torch.randint(w.B, (1,), generator=g)); h = int(torch.randint(w.H, (1,), generator=g))
        i = int(torch.randint(w.Tm, (1,), generator=g))
        c = int(pat.row_cnt[b, h, i])
        assert torch.equal(pat.row_idx[b, h, i, :c].long(), torch.nonzero(m[b, h, i]).flatten())


@pytest.mark.parametrize("w", [wl.WAN13_95, wl.WAN14_95], ids=lambda w: w.name)
def test_wan_like_layers_sampled(w):
    print(f"workload {w.name}: B={w.B} H={w.H} N={w.N} d={w.d}", flush=True)
    q, k, v, do = wl.make_inputs(w, seed=0, device=dev())
    k_cnt, pat, pbar, o, lse, dq, dk, dv = _run_path(w, q, k, v, do)
    _properties(w, pat, o, lse, dq, dk, dv, k_cnt)
    density = float(pat.mask.float().mean())
    print(f"  block sparsity {1 - density:.4f}", flush=True)
    assert 0.90 < 1 - density < 0.95
    heads = [(0, 0), (0, w.H - 1)]
    for (b, h) in heads:
        # mask protocol on the whole head
        ref_pbar = orc.pooled_map(f64(q[b, h]), f64(k[b, h]))
        r = mask_protocol(pat.mask[b, h].cpu().numpy(), pbar[b, h].cpu().numpy(), ref_pbar, k_cnt, w.top_p)
        print(f"  head ({b},{h}) mask protocol: {r}", flush=True)
        assert r["stage1_max_rel"] <= 1e-5 and r["stage2_unexplained"] == 0 and r["stage3_unexplained"] == 0
        # sampled blocks: first, a Top-p-bound (longest) row, the ragged last ones; hottest and last key blocks
        rc = pat.row_cnt[b, h].cpu().numpy(); cc = pat.col_cnt[b, h].cpu().numpy()
        q_blocks = sorted({0, int(rc.argmax()), w.Tm // 2, w.Tm - 1})
        kv_blocks = sorted({int(cc.argmax()), w.Tn // 3, w.Tn - 1})
        _check_head_samples(w, b, h, q, k, v, do, pat, o, lse, dq, dk, dv, q_blocks, kv_blocks)


def test_head_dim_64_layer_sampled():
    """The d = 64 instantiations of every kernel on a layer long enough for many tiles per row and column,
    batch 2, with a ragged tail (20,010 = 156 * 128 + 42 = 312 * 64 + 42)."""
    w = wl.Workload("d64-20k", 2, 3, 20010, 64, 0.05, 0.8, "lowrank", True)
    print(f"workload {w.name}: B={w.B} H={w.H} N={w.N} d={w.d}", flush=True)
    q, k, v, do = wl.make_inputs(w, seed=0, device=dev())
    k_cnt, pat, pbar, o, lse, dq, dk, dv = _run_path(w, q, k, v, do)
    _properties(w, pat, o, lse, dq, dk, dv, k_cnt)
    b, h = 1, 2
    ref_pbar = orc.pooled_map(f64(q[b, h]), f64(k[b, h]))
    r = mask_protocol(pat.mask[b, h].cpu().numpy(), pbar[b, h].cpu().numpy(), ref_pbar, k_cnt, w.top_p)
    print(f"  head ({b},{h}) mask protocol: {r}", flush=True)
    assert r["stage1_max_rel"] <= 1e-5 and r["stage2_unexplained"] == 0 and r["stage3_unexplained"] == 0
    rc = pat.row_cnt[b, h].cpu().numpy(); cc = pat.col_cnt[b, h].cpu().numpy()
    _check_head_samples(w, b, h, q, k, v, do, pat, o, lse, dq, dk, dv,
                        q_blocks=sorted({0, int(rc.argmax()), w.Tm - 1}), kv_blocks=sorted({int(cc.argmax()), w.Tn - 1}))


STRESS_SETTINGS = [(kf, p) for kf in (0.02, 0.05, 0.10) for p in (0.5, 0.8, 0.95)]


def test_mask_stress_sweep():
    """Near-uniform rows (thousands of near-ties) and sink-dominated rows: the mask must still equal
    the oracle's selection on the exported scores; flips are counted per setting."""
    w = wl.MASK_STRESS
    print(f"workload {w.name}: B={w.B} H={w.H} N={w.N} d={w.d}", flush=True)
    q, k, v, do = wl.make_inputs(w, seed=0, device=dev())
    ref_pbar = {(b, h): orc.pooled_map(f64(q[b, h]), f64(k[b, h])) for (b, h) in [(0, 0), (1, 7)]}
    for si, (kf, p) in enumerate(STRESS_SETTINGS):
        k_cnt, pat, pbar, o, lse, dq, dk, dv = _run_path(w, q, k, v, do, kf, p)
        _properties(w, pat, o, lse, dq, dk, dv, k_cnt)
        tot = {}
        for (b, h), rp in ref_pbar.items():
            r = mask_protocol(pat.mask[b, h].cpu().numpy(), pbar[b, h].cpu().numpy(), rp, k_cnt, p)
            assert r["stage1_max_rel"] <= 1e-5 and r["stage2_unexplained"] == 0 and r["stage3_unexplained"] == 0, r
            for key, val in r.items():
                if key.startswith("stage") and key != "stage1_max_rel":
                    tot[key] = tot.get(key, 0) + val
        print(f"  k={kf} p={p}: k_cnt={k_cnt} density={float(pat.mask.float().mean()):.4f} flips={tot}", flush=True)
        if si in (1, 8):      # attention spot checks on two settings (sparse-ish and dense-ish)
            b, h = 1, 7
            cc = pat.col_cnt[b, h].cpu().numpy()
            _check_head_samples(w, b, h, q, k, v, do, pat, o, lse, dq, dk, dv,
                                q_blocks=[0, 1, w.Tm - 1], kv_blocks=[0, int(cc[1:].argmax()) + 1])
