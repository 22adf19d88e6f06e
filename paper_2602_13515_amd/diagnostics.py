"""Masking diagnostics on top of the C calls: the error of a masking rule against full attention with its
dropped / renormalisation split (Sec. 3.1, the relative L1 metric of Sec. 3.2), Top-k-only and Top-p-only
masking (Sec. 2.2) as special cases of the hybrid rule, and the calibration of k% / p% to a target sparsity
(appendix on hyper-parameters).  Buffers come from PyTorch; every array operation runs in the HIP kernels;
only the handful of scalars that steer a bisection are read back to the host.
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import torch

from . import binding as _b


def _mask(q, k, k_frac: float, top_p: float, scale: float, pattern: Optional[_b.Pattern] = None,
          workspace: Optional[torch.Tensor] = None) -> _b.Pattern:
    B, H, N, _ = q.shape
    pattern = pattern if pattern is not None else _b.alloc_pattern(B, H, N, q.device)
    if workspace is None:
        workspace = torch.empty(_b.spa2_mask_workspace_bytes(q), dtype=torch.uint8, device=q.device)
    _b.spa2_mask(q, k, _b.spa2_topk_blocks(float(k_frac), -(-N // _b.BKV)), float(top_p), scale, pattern, None, workspace)
    return pattern


def block_sparsity(pattern: _b.Pattern) -> float:
    """Fraction of tiles the pattern skips."""
    total = pattern.mask.shape[-1] * pattern.row_cnt.numel()
    return 1.0 - float(pattern.row_cnt.sum(dtype=torch.int64).item()) / total


def masking_error(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, k_frac: float, top_p: float,
                  scale: Optional[float] = None) -> Dict[str, torch.Tensor]:
    """Error of the masking rule (k_frac, top_p) on (q, k, v) against full attention, per (batch, head).

    k_frac = 0 gives Top-p-only masking and top_p = 0 Top-k-only masking.  Returns float64 [B, H] tensors:
    `rel_l1` = sum|o - o_s| / sum|o|, `dropped` and `renorm` (the two parts of Sec. 3.1, same normaliser),
    `tau` (mean retained attention mass per row), and the scalar `sparsity`."""
    B, H, N, d = q.shape
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    dev = q.device
    pat = _mask(q, k, k_frac, top_p, scale)
    full = _b.alloc_pattern(B, H, N, dev, columns=False)
    _b.spa2_pattern_full(q, full)
    o_s, o_f = torch.empty_like(q), torch.empty_like(q)
    lse_s = torch.empty((B, H, N), dtype=torch.float32, device=dev)
    lse_f = torch.empty_like(lse_s)
    _b.spa2_fwd(q, k, v, pat, scale, o_s, lse_s)
    _b.spa2_fwd(q, k, v, full, scale, o_f, lse_f)
    out = torch.empty((B, H, 5), dtype=torch.float64, device=dev)
    ws = torch.empty(max(_b.spa2_error_workspace_bytes(q), 16), dtype=torch.uint8, device=dev)
    _b.spa2_error_terms(o_s, o_f, lse_s, lse_f, out, ws)
    ref = out[..., 1]
    return {"rel_l1": out[..., 0] / ref, "dropped": out[..., 2] / ref, "renorm": out[..., 3] / ref,
            "tau": out[..., 4] / N, "sparsity": block_sparsity(pat)}


def calibrate(q: torch.Tensor, k: torch.Tensor, target_sparsity: float, *, k_frac: Optional[float] = None,
              top_p: Optional[float] = None, scale: Optional[float] = None, tol: float = 2e-3,
              max_iter: int = 24) -> Dict[str, float]:
    """Bisection on one of the two masker parameters, the other held fixed, until the block sparsity of the
    pattern on (q, k) is within `tol` of `target_sparsity` (sparsity falls monotonically in both).  Give
    `k_frac` to search top_p, or `top_p` to search k_frac.  Uses spa2_mask only; one scalar per step is read
    back.  Returns the parameters, the sparsity reached and the number of masker calls."""
    if (k_frac is None) == (top_p is None):
        raise ValueError("fix exactly one of k_frac / top_p; the other one is searched")
    B, H, N, d = q.shape
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    pat = _b.alloc_pattern(B, H, N, q.device, columns=False)
    ws = torch.empty(_b.spa2_mask_workspace_bytes(q), dtype=torch.uint8, device=q.device)
    search_p = top_p is None

    def sparsity_at(x: float) -> float:
        kf, tp = (k_frac, x) if search_p else (x, top_p)
        if kf <= 0.0 and tp <= 0.0:
            return 1.0 - 1.0 / pat.mask.shape[-1]          # the rule keeps one block per row at least
        return block_sparsity(_mask(q, k, kf, tp, scale, pat, ws))

    lo, hi = 0.0, 1.0                                       # sparsity(lo) >= target >= sparsity(hi)
    calls = 0
    best = (hi, sparsity_at(hi)); calls += 1
    s_lo = sparsity_at(lo); calls += 1
    if s_lo < target_sparsity:                              # even the smallest setting is too dense
        best = (lo, s_lo)
    else:
        for _ in range(max_iter):
            mid = 0.5 * (lo + hi)
            s = sparsity_at(mid); calls += 1
            if abs(s - target_sparsity) < abs(best[1] - target_sparsity):
                best = (mid, s)
            if abs(s - target_sparsity) <= tol:
                break
            if s > target_sparsity:
                lo = mid
            else:
                hi = mid
    x, s = best
    return {"k_frac": float(k_frac if search_p else x), "top_p": float(x if search_p else top_p),
            "sparsity": float(s), "mask_calls": calls}
