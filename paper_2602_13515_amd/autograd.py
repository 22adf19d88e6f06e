"""`O = SpargeAttn2(Q, K, V, k%, p%)` (Sec. 4.3, Alg. 1) as a differentiable PyTorch operator.

A thin `torch.autograd.Function` over the three C calls: `spa2_mask` builds the block pattern from
Q and K, `spa2_fwd` runs the block-sparse attention, `spa2_bwd` returns dQ, dK, dV with the pattern
held constant (no gradient flows through the pooled scores, as in Alg. 2 where the mask is an
input of the attention call).  PyTorch allocates the buffers; every step runs in the HIP kernels.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import torch

from . import binding as _b


def _like(x: torch.Tensor) -> torch.Tensor:
    return torch.empty_strided(x.shape, x.stride(), dtype=x.dtype, device=x.device)


def _match(x: torch.Tensor, ref: torch.Tensor) -> torch.Tensor:
    """x with ref's strides (the kernels take one stride triple for all token tensors of a call)."""
    if x.stride() == ref.stride():
        return x
    y = _like(ref)
    y.copy_(x)
    return y


def _check_inputs(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor) -> None:
    for name, t in (("q", q), ("k", k), ("v", v)):
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU: the operator has no CPU path")
        if t.dtype != torch.bfloat16 or t.dim() != 4:
            raise ValueError(f"{name} must be a bf16 [B, H, N, d] view")
    if k.shape != q.shape or v.shape != q.shape:
        raise ValueError("self-attention: q, k, v share one shape")
    if q.stride(3) != 1:
        raise ValueError("the head dimension must be contiguous")


def build_pattern(q: torch.Tensor, k: torch.Tensor, k_frac: float, top_p: float,
                  scale: Optional[float] = None) -> _b.Pattern:
    """Hybrid Top-k + Top-p block pattern of (q, k) (Sec. 4.1; Alg. 1 steps 4-6)."""
    B, H, N, d = q.shape
    scale = 1.0 / math.sqrt(d) if scale is None else float(scale)
    k = _match(k, q)
    pat = _b.alloc_pattern(B, H, N, q.device)
    ws = torch.empty(_b.spa2_mask_workspace_bytes(q), dtype=torch.uint8, device=q.device)
    k_cnt = _b.spa2_topk_blocks(float(k_frac), -(-N // _b.BKV))
    _b.spa2_mask(q, k, k_cnt, float(top_p), scale, pat, None, ws)
    return pat


_side_streams = {}


def _side_stream(device: torch.device) -> torch.cuda.Stream:
    """One extra stream per device (default priority), made on first use, for `overlap_backward`."""
    key = torch.device(device).index
    if key not in _side_streams:
        _side_streams[key] = torch.cuda.Stream(device=device)
    return _side_streams[key]


def backward_two_streams(q, k, v, o, d_o, lse, pattern, scale, dq, dk, dv, workspace, o_res=None) -> None:
    """The backward pass as its three stage calls, with the dK/dV kernel on the current stream and the dQ kernel
    on a side stream at the same time.  Both read D, which the first call writes; they write different tensors,
    so the results are the bits `spa2_bwd` gives.  The two kernels fill each other's idle slots; measured on the
    75,600-token layer this is worth 0.2 ms of a 35 ms step (1.2 ms of 27 when only the backward pass runs in a
    loop)."""
    cur, side = torch.cuda.current_stream(q.device), _side_stream(q.device)
    _b.spa2_bwd_delta(o, d_o, workspace, o_res)
    fork = torch.cuda.Event()
    fork.record(cur)
    side.wait_event(fork)
    with torch.cuda.stream(side):
        _b.spa2_bwd_dq(q, k, v, d_o, lse, pattern, scale, dq, workspace)
    _b.spa2_bwd_dkdv(q, k, v, d_o, lse, pattern, scale, dk, dv, workspace)
    join = torch.cuda.Event()
    join.record(side)
    cur.wait_event(join)
    for t in (q, k, v, d_o, lse, dq, workspace):       # the caching allocator must not hand these out early
        t.record_stream(side)


class _SpargeAttn2(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, scale, pattern, overlap_backward=False):
        k, v = _match(k, q), _match(v, q)
        B, H, N, _ = q.shape
        o, o_res = _like(q), _like(q)
        lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
        ws_f = torch.empty(_b.spa2_fwd_workspace_bytes(q), dtype=torch.uint8, device=q.device)   # long rows split
        _b.spa2_fwd(q, k, v, pattern, scale, o, lse, o_res, ws_f)
        ctx.save_for_backward(q, k, v, o, o_res, lse)
        ctx.pattern, ctx.scale, ctx.overlap = pattern, scale, bool(overlap_backward)
        return o

    @staticmethod
    def backward(ctx, d_o):
        q, k, v, o, o_res, lse = ctx.saved_tensors
        d_o = _match(d_o.to(torch.bfloat16), q)
        dq, dk, dv = _like(q), _like(q), _like(q)
        ws = torch.empty(_b.spa2_bwd_workspace_bytes(q), dtype=torch.uint8, device=q.device)
        if ctx.overlap:
            backward_two_streams(q, k, v, o, d_o, lse, ctx.pattern, ctx.scale, dq, dk, dv, ws, o_res)
        else:
            _b.spa2_bwd(q, k, v, o, d_o, lse, ctx.pattern, ctx.scale, dq, dk, dv, ws, o_res)
        return dq, dk, dv, None, None, None


def sparge_attn2(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, k_frac: float, top_p: float,
                 scale: Optional[float] = None, pattern: Optional[_b.Pattern] = None,
                 return_pattern: bool = False, overlap_backward: bool = False):
    """Block-sparse attention on the blocks that the hybrid Top-k + Top-p rule selects.

    q, k, v: bf16 [B, H, N, d] views, d in {64, 128}, d contiguous; a [B, N, H, d] tensor is passed as
    `x.permute(0, 2, 1, 3)` without a copy.  k_frac, top_p in [0, 1].  `pattern`, when given, is used instead
    of building one from (q, k).  `overlap_backward` runs the two backward kernels at the same time on two
    streams (same results).  Returns O with q's shape and strides (and the pattern on request)."""
    _check_inputs(q, k, v)
    scale = 1.0 / math.sqrt(q.shape[-1]) if scale is None else float(scale)
    if pattern is None:
        with torch.no_grad():
            pattern = build_pattern(q.detach(), k.detach(), k_frac, top_p, scale)
    o = _SpargeAttn2.apply(q, k, v, scale, pattern, overlap_backward)
    return (o, pattern) if return_pattern else o


class SpargeAttn2(torch.nn.Module):
    """Attention core with fixed k% and p% (the appendix on hyper-parameters uses Top-k = 0.03 with Top-p = 0.2 or
    0.16 for about 95 % sparsity)."""

    def __init__(self, k_frac: float, top_p: float, scale: Optional[float] = None):
        super().__init__()
        self.k_frac, self.top_p, self.scale = float(k_frac), float(top_p), scale

    def forward(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor) -> torch.Tensor:
        return sparge_attn2(q, k, v, self.k_frac, self.top_p, self.scale)

    def extra_repr(self) -> str:
        return f"k_frac={self.k_frac}, top_p={self.top_p}"
