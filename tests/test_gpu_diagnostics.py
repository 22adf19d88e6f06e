"""Error decomposition of Sec. 3.1 from the HIP kernels against the oracle's row-by-row version, the
qualitative ordering of the three masking rules on uniform and skewed rows (Case 1 of Sec. 3.2), and the
k% / p% calibration."""
import math

import numpy as np
import pytest
import torch

import paper_2602_13515_amd as spa2
from oracle import spa2_oracle as orc
from paper_2602_13515_amd import workloads as wl

from gpu_util import dev, f64

pytestmark = pytest.mark.gpu


def _terms(q, k, v, pat):
    B, H, N, d = q.shape
    scale = 1.0 / math.sqrt(d)
    full = spa2.alloc_pattern(B, H, N, q.device, columns=False)
    spa2.spa2_pattern_full(q, full)
    o_s, o_f = torch.empty_like(q), torch.empty_like(q)
    lse_s = torch.empty((B, H, N), dtype=torch.float32, device=q.device); lse_f = torch.empty_like(lse_s)
    spa2.spa2_fwd(q, k, v, pat, scale, o_s, lse_s)
    spa2.spa2_fwd(q, k, v, full, scale, o_f, lse_f)
    out = torch.full((B, H, 5), float("nan"), dtype=torch.float64, device=q.device)
    ws = torch.empty(max(spa2.spa2_error_workspace_bytes(q), 16), dtype=torch.uint8, device=q.device)
    spa2.spa2_error_terms(o_s, o_f, lse_s, lse_f, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), o_s, o_f, lse_s, lse_f


@pytest.mark.parametrize("d", [64, 128])
def test_error_terms_match_oracle(d):
    w = wl.Workload("diag", 1, 2, 700, d, 0.2, 0.5, "gaussian", False)      # several chunks of rows, ragged tail
    q, k, v = (t.to(dev()) for t in wl.make_inputs(w, seed=2)[:3])
    pat = spa2.build_pattern(q, k, w.k_frac, w.top_p)
    got, o_s, o_f, lse_s, lse_f = _terms(q, k, v, pat)
    mask = pat.mask.cpu().numpy()
    for h in range(w.H):
        ref = np.array(orc.error_sums(f64(q[0, h]), f64(k[0, h]), f64(v[0, h]), mask[0, h]))
        # outputs are bf16: 2^-9 relative per element, well inside 1 % on L1 norms of thousands of elements
        assert np.allclose(got[0, h, :4], ref[:4], rtol=1e-2), (got[0, h], ref)
        assert abs(got[0, h, 4] - ref[4]) <= 1e-3 * ref[4]
        # the kernel's own reduction, re-done in fp64 on the host from the very same device outputs
        os_, of_ = f64(o_s[0, h]), f64(o_f[0, h])
        tau = np.exp(f64(lse_s[0, h]) - f64(lse_f[0, h]))[:, None]
        host = [np.abs(of_ - os_).sum(), np.abs(of_).sum(), np.abs(of_ - tau * os_).sum(), np.abs((tau - 1) * os_).sum(), tau.sum()]
        assert np.allclose(got[0, h], host, rtol=2e-5), (got[0, h], host)


def test_error_terms_are_deterministic_and_zero_for_the_full_pattern():
    w = wl.Workload("diag2", 2, 2, 520, 128, 0.3, 0.3, "lowrank", False)
    q, k, v = (t.to(dev()) for t in wl.make_inputs(w, seed=4)[:3])
    full = spa2.alloc_pattern(w.B, w.H, w.N, dev(), columns=False)
    spa2.spa2_pattern_full(q, full)
    got = _terms(q, k, v, full)[0]
    assert (got[..., 0] == 0).all() and (got[..., 2] == 0).all() and (got[..., 3] == 0).all()
    assert np.allclose(got[..., 4], w.N)
    pat = spa2.build_pattern(q, k, w.k_frac, w.top_p)
    a = _terms(q, k, v, pat)[0]; b = _terms(q, k, v, pat)[0]
    assert np.array_equal(a, b)


def test_masking_rules_order_as_in_case_1():
    """Uniform rows: at equal sparsity Top-k loses a fixed share of the mass while Top-p keeps its target, and
    skewed (sink) rows turn the order around: there Top-p stops after the sink block, Top-k keeps more context
    (Sec. 3.2, Case 1).  The hybrid rule is never worse than the better of the two by construction (its mask
    contains both)."""
    w = wl.Workload("stress-small", 1, 2, 4096, 128, 0.05, 0.8, "stress", False)
    q, k, v = (t.to(dev()) for t in wl.make_inputs(w, seed=0)[:3])
    topk = spa2.masking_error(q, k, v, 0.10, 0.0)
    topp = spa2.masking_error(q, k, v, 0.0, 0.6)
    both = spa2.masking_error(q, k, v, 0.10, 0.6)
    for r in (topk, topp, both):
        assert torch.isfinite(r["rel_l1"]).all() and (r["tau"] > 0).all() and (r["tau"] <= 1 + 1e-6).all()
    # the hybrid mask is a superset of either mask: it retains at least as much mass and is denser
    assert (both["tau"] >= topk["tau"] - 1e-6).all() and (both["tau"] >= topp["tau"] - 1e-6).all()
    assert both["sparsity"] <= min(topk["sparsity"], topp["sparsity"]) + 1e-9
    assert (both["rel_l1"] <= torch.maximum(topk["rel_l1"], topp["rel_l1"]) + 1e-3).all()
    print("rel L1  top-k %s  top-p %s  hybrid %s" % (topk["rel_l1"].flatten().tolist(), topp["rel_l1"].flatten().tolist(),
                                                    both["rel_l1"].flatten().tolist()))


def test_calibration_hits_the_target_sparsity():
    w = wl.Workload("cal", 1, 2, 8192, 128, 0.05, 0.8, "lowrank", False)
    q, k = (t.to(dev()) for t in wl.make_inputs(w, seed=0)[:2])
    r = spa2.calibrate(q, k, 0.90, k_frac=0.03)
    assert abs(r["sparsity"] - 0.90) <= 2e-3 and 0.0 < r["top_p"] < 1.0 and r["mask_calls"] <= 26, r
    r2 = spa2.calibrate(q, k, 0.90, top_p=0.2)
    assert abs(r2["sparsity"] - 0.90) <= 5e-3 and 0.0 < r2["k_frac"] < 1.0, r2     # k moves in steps of one block
    with pytest.raises(ValueError):
        spa2.calibrate(q, k, 0.9)
