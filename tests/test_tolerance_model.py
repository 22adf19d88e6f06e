"""Where the parity bars on O, dQ, dK, dV come from (CPU only; the oracle plus numpy roundings).

The benchmark definition asks for max-abs <= 2e-2 and mean-abs <= 2e-3 against the fp64 oracle.  The design
fixes four roundings that no kernel schedule can avoid: the attention weights P and the score gradients dS
are rounded to bf16 before the second matrix product, O is stored in bf16 (plus an optional bf16 residual)
and feeds D = rowsum(dO * O), and every output is stored in bf16.  This file applies exactly those
roundings, and nothing else, to an otherwise exact fp64 evaluation of the same formulas, on the inputs where
tests/gpu_util.py::assert_close is given a wider bar than the plain one, and checks that

  * the plain bar is not reachable there (the emulated worst element is above 2e-2), so widening is needed;
  * each widened bar is of the size of the roundings' own worst element: within a factor 2 of the emulated worst
    (2.5 for dQ at the largest shape).  The emulation is one realisation of the roundings (on which side of a
    rounding boundary a value of dS falls depends on the last bits of D), and single large entries of dS dominate
    the worst element, so its worst element estimates the size of the tail; it is not a bound;
  * wherever values are of order one (small Gaussian problems) the emulation stays far inside the plain bar.

No number in this file comes from the GPU.  The emulation is written here from the formulas of the oracle's
backward pass (dV = P^T dO, dP = dO V^T, D = rowsum(dO * O), dS = P * (dP - D), dQ = dS K scale,
dK = dS^T Q scale; Sec. 4.3 names the pass) and shares no code with the HIP library.
"""
import math

import numpy as np
import pytest

from oracle import spa2_oracle as orc
from paper_2602_13515_amd import workloads as wl

# the bars of tests/gpu_util.py::assert_close, restated (test_bars_match_gpu_util keeps them in step)
MAX_ABS, MEAN_ABS = 2e-2, 2e-3
ROW_REL, MEAN_REL = 2.0 ** -7, 2.0 ** -8
LOWRANK_MAX_ABS = 5e-2


def bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value (ties to even), returned as float64."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def f64(t):
    return t.double().numpy()


def emulate(q, k, v, do, mask, q_blocks, residual=True):
    """The backward formulas in fp64 with the four design roundings, over the given query blocks.
    Returns (O, dQ) rows of those blocks (bf16 values) and the fp64 sums dK, dV of their contributions
    (not yet rounded: a key block is complete only when every query block of its column was visited)."""
    n, d = q.shape
    scale = 1.0 / math.sqrt(d)
    o = np.zeros((n, d)); dq = np.zeros((n, d)); dk = np.zeros((n, d)); dv = np.zeros((n, d))
    for i in q_blocks:
        r0, r1 = i * 128, min(n, (i + 1) * 128)
        cols = np.concatenate([np.arange(j * 64, min(n, (j + 1) * 64)) for j in np.flatnonzero(mask[i])])
        s = (q[r0:r1] @ k[cols].T) * scale
        m = s.max(1, keepdims=True)
        e = bf16(np.exp(s - m))                            # P of the forward pass: bf16 before P V
        o_i = (e @ v[cols]) / e.sum(1, keepdims=True)      # numerator and denominator over the same rounded P
        o_b = bf16(o_i)
        o_used = o_b + (bf16(o_i - o_b) if residual else 0.0)
        lse = m + np.log(e.sum(1, keepdims=True))          # LSE carries the row sum of the rounded P
        p = np.exp(s - lse)                                # backward: P recomputed from LSE in fp32
        dd = (do[r0:r1] * o_used).sum(1, keepdims=True)
        ds = bf16(p * (do[r0:r1] @ v[cols].T - dd))        # dS: bf16 before dS K and dS^T Q
        o[r0:r1] = o_b
        dq[r0:r1] = bf16((ds @ k[cols]) * scale)
        np.add.at(dk, cols, ds.T @ q[r0:r1])
        np.add.at(dv, cols, bf16(p).T @ do[r0:r1])         # P: bf16 before P^T dO
    return o, dq, dk * scale, dv


def bars(ref, max_abs=MAX_ABS):
    rowmax = np.abs(ref).max(-1, keepdims=True)
    return np.maximum(max_abs, ROW_REL * rowmax), max(MEAN_ABS, MEAN_REL * float(np.abs(ref).mean()))


def report(name, got, ref, max_abs=MAX_ABS):
    err = np.abs(got - ref)
    tol, mean_bar = bars(ref, max_abs)
    over_plain = int((err > MAX_ABS).sum())
    print(f"  {name}: emulated max {err.max():.4f} mean {err.mean():.5f}; elements above 2e-2: {over_plain} of {err.size}; "
          f"largest bar used {tol.max():.4f}, mean bar {mean_bar:.5f}", flush=True)
    return err, tol, mean_bar, over_plain


def test_bars_match_gpu_util():
    import gpu_util
    assert (gpu_util.MAX_ABS, gpu_util.MEAN_ABS, gpu_util.BF16_ULP_REL) == (MAX_ABS, MEAN_ABS, ROW_REL)
    assert gpu_util.LOWRANK_MAX_ABS == LOWRANK_MAX_ABS


def test_gaussian_inputs_stay_inside_the_plain_bar():
    """Values of order one: every rounding is far below the plain bar (the small parity cases keep 2e-2 / 2e-3)."""
    w = wl.Workload("g", 1, 1, 1000, 128, 0.25, 0.9, "gaussian", True)
    q, k, v, do = (f64(t)[0, 0] for t in wl.make_inputs(w, seed=1))
    mask, _ = orc.block_mask(q, k, orc.topk_blocks(w.k_frac, w.Tn), w.top_p)
    r_dq, r_dk, r_dv, r_o, _ = orc.attention_bwd_gather(q, k, v, mask, do)
    o, dq, dk, dv = emulate(q, k, v, do, mask, range(w.Tm))
    for name, got, ref in (("O", o, r_o), ("dQ", dq, r_dq), ("dK", bf16(dk), r_dk), ("dV", bf16(dv), r_dv)):
        err, _, _, over = report(name, got, ref)
        assert over == 0 and err.max() <= MAX_ABS / 2 and err.mean() <= MEAN_ABS / 2


def test_small_lowrank_inputs_need_and_meet_the_5e2_bar():
    """N = 1281, d = 64, rank-4 scale-2 component (the block-edge sweep's low-rank case): dS, rounded to bf16,
    multiplies queries and keys of magnitude 8-10.  The plain 2e-2 is exceeded by the roundings alone; the
    5e-2 given to dQ and dK on low-rank inputs is attainable and within 2x of the emulated worst element."""
    N, d = 1281, 64
    w = wl.Workload("edge", 1, 2, N, d, 0.3, 0.6, "lowrank", True)
    qq, kk, vv, dd = wl.make_inputs(w, seed=100 + N)
    worst = {"dQ": 0.0, "dK": 0.0}
    for h in range(w.H):
        q, k, v, do = (f64(t)[0, h] for t in (qq, kk, vv, dd))
        mask, _ = orc.block_mask(q, k, orc.topk_blocks(w.k_frac, w.Tn), w.top_p)
        r_dq, r_dk, r_dv, r_o, _ = orc.attention_bwd_gather(q, k, v, mask, do)
        o, dq, dk, dv = emulate(q, k, v, do, mask, range(w.Tm), residual=False)
        print(f"head {h}: max|Q| {np.abs(q).max():.1f} max|K| {np.abs(k).max():.1f}", flush=True)
        for name, got, ref in (("dQ", dq, r_dq), ("dK", bf16(dk), r_dk)):
            err, tol, mean_bar, _ = report(name, got, ref, LOWRANK_MAX_ABS)
            assert err.mean() <= mean_bar / 2
            # elements whose bar is the 5e-2 floor (rows of small magnitude): worst emulated error among them
            floor_rows = (tol == LOWRANK_MAX_ABS)[:, 0]
            worst[name] = max(worst[name], float(err[floor_rows].max()))
            assert (err <= 1.25 * tol).all()
        for name, got, ref in (("O", o, r_o), ("dV", bf16(dv), r_dv)):     # these keep the 2e-2 floor
            err, tol, mean_bar, over = report(name, got, ref)
            assert (err <= tol).all() and err.mean() <= mean_bar
    print(f"worst emulated element under the 5e-2 floor: {worst}", flush=True)
    for name, e in worst.items():
        assert e > MAX_ABS, f"{name}: the plain bar would do, drop the widening"
        assert LOWRANK_MAX_ABS / 2 <= e <= LOWRANK_MAX_ABS * 1.25, (name, e)


@pytest.fixture(scope="module")
def wan_head():
    """Head 0 of the 32,760-token low-rank layer with its oracle mask (k = 5 %, p = 0.8)."""
    w = wl.WAN13_95
    q, k, v, do = (f64(t) for t in wl.head_inputs(w, 0, 0, seed=0))
    mask, _ = orc.block_mask(q, k, orc.topk_blocks(w.k_frac, w.Tn), w.top_p)
    return w, q, k, v, do, mask


def test_hot_key_block_needs_and_meets_the_row_scaled_bar(wan_head):
    """The key block that most query blocks select collects |dK| of 20 and more per element: bf16 numbers are
    0.125 apart there, so an absolute 2e-2 cannot hold for the stored result.  The bar max(2e-2, 2^-7 x the row's
    largest reference value) holds for the emulation and is within 2x of its error at the worst element; the mean
    bar max(2e-3, 2^-8 x mean|ref|) likewise."""
    w, q, k, v, do, mask = wan_head
    j = int(mask.sum(0).argmax())
    rows = [int(i) for i in np.flatnonzero(mask[:, j])]
    c0, c1 = j * 64, min(w.N, (j + 1) * 64)
    _, r_dk, r_dv, _, _ = orc.attention_bwd_gather(q, k, v, mask, do, q_blocks=rows)
    _, _, dk, dv = emulate(q, k, v, do, mask, rows)
    print(f"key block {j}: selected by {len(rows)} query blocks; max|dK ref| {np.abs(r_dk[c0:c1]).max():.1f}", flush=True)
    err, tol, mean_bar, over = report("dK", bf16(dk[c0:c1]), r_dk[c0:c1])
    assert over > 0 and err.max() > 2 * MAX_ABS, "the plain bar would do: drop the row scaling"
    assert err.mean() > MEAN_ABS, "the plain mean bar would do: drop its scaling"
    assert (err <= tol).all() and err.mean() <= mean_bar
    # of the right size: the largest ratio of an element's error to its bar is at least 1/2, and so is the mean's
    print(f"  largest error / bar over the block: {(err / tol).max():.2f}; mean error / mean bar {err.mean() / mean_bar:.2f}", flush=True)
    assert (err / tol).max() >= 0.5 and err.mean() >= 0.5 * mean_bar
    err_v, tol_v, mean_bar_v, _ = report("dV", bf16(dv[c0:c1]), r_dv[c0:c1])
    assert (err_v <= tol_v).all() and err_v.mean() <= mean_bar_v


def test_long_layer_dq_needs_and_meets_the_5e2_bar():
    """dQ on the 75,600-token low-rank layer (head 39, every 12th query block, Top-p-bound rows of several hundred
    tiles included): rows of dQ stay of order one, so the row-scaled bar does not apply, yet dS in bf16 times keys of
    magnitude ~10 moves single elements past 2e-2.  The 5e-2 given to dQ there is within 2.5x of the emulated worst
    element over these 50 blocks (the worst over all 23,640 blocks of the layer lies further out in the same tail)."""
    w = wl.WAN14_95
    q, k, v, do = (f64(t) for t in wl.head_inputs(w, 0, 39, seed=0))
    mask, _ = orc.block_mask(q, k, orc.topk_blocks(w.k_frac, w.Tn), w.top_p)
    blocks = list(range(0, w.Tm, 12))
    r_dq, _, _, r_o, _ = orc.attention_bwd_gather(q, k, v, mask, do, q_blocks=blocks)
    o, dq, _, _ = emulate(q, k, v, do, mask, blocks)
    rows = np.concatenate([np.arange(i * 128, min(w.N, (i + 1) * 128)) for i in blocks])
    print(f"{len(blocks)} query blocks, row lengths {int(mask.sum(1)[blocks].min())}..{int(mask.sum(1)[blocks].max())} tiles; "
          f"max|dQ ref| {np.abs(r_dq[rows]).max():.2f}, max|K| {np.abs(k).max():.1f}", flush=True)
    err, tol, mean_bar, over = report("dQ", dq[rows], r_dq[rows], LOWRANK_MAX_ABS)
    assert (err <= tol).all() and err.mean() <= mean_bar / 2
    assert err.max() > MAX_ABS, "the plain bar would do: drop the widening"
    assert LOWRANK_MAX_ABS <= 2.5 * err.max(), err.max()
    err_o, _, _, over_o = report("O", o[rows], r_o[rows])
    assert over_o == 0 and err_o.mean() <= MEAN_ABS / 2
