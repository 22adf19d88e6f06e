"""Adapting a model to SpargeAttention2 by velocity distillation (Sec. 4.2; Alg. 2), on a toy scale.

The paper fine-tunes video diffusion models whose weights are not available here; what can be exercised
without them is the training step itself: a frozen teacher with full attention, a student that shares its
initialisation and differs only in the attention operator, identical noisy inputs x_t = t x_1 + (1 - t) x_0
for both, and the loss ||u_sparse - u_full||^2 back-propagated through the block-sparse backward kernels.
`ToyBlock` is one pre-norm attention block that stands in for the velocity network.
"""
from __future__ import annotations

import copy
from typing import Callable, Dict, Iterable, Optional, Tuple

import torch

from . import binding as _b
from .autograd import sparge_attn2


class ToyBlock(torch.nn.Module):
    """x -> x + proj(attention(norm(x))): fp32 parameters, bf16 attention on [B, N, H, d] activations that reach
    the kernels as permuted views (no copy).  `k_frac`, `top_p` None means full attention (the teacher)."""

    def __init__(self, dim: int, heads: int, k_frac: Optional[float] = None, top_p: Optional[float] = None):
        super().__init__()
        assert dim % heads == 0 and dim // heads in (64, 128)
        self.heads, self.k_frac, self.top_p = heads, k_frac, top_p
        self.norm = torch.nn.LayerNorm(dim)
        self.qkv = torch.nn.Linear(dim, 3 * dim)
        self.proj = torch.nn.Linear(dim, dim)
        self._full = None                     # the all-ones pattern, built once per input shape

    def _attention(self, q, k, v):
        if self.k_frac is not None:
            return sparge_attn2(q, k, v, self.k_frac, self.top_p)
        B, H, N, _ = q.shape
        if self._full is None or self._full.mask.shape[:3] != (B, H, -(-N // _b.BQ)) or self._full.mask.device != q.device:
            self._full = _b.alloc_pattern(B, H, N, q.device)
            _b.spa2_pattern_full(q.detach(), self._full)
        return sparge_attn2(q, k, v, 0.0, 0.0, pattern=self._full)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        B, N, C = x.shape
        qkv = self.qkv(self.norm(x)).to(torch.bfloat16).view(B, N, 3, self.heads, C // self.heads)
        q, k, v = (qkv[:, :, i].permute(0, 2, 1, 3) for i in range(3))         # [B, H, N, d] views
        o = self._attention(q, k, v)                                            # strides of q
        return x + self.proj(o.permute(0, 2, 1, 3).reshape(B, N, C).float())


def make_student(teacher: ToyBlock, k_frac: float, top_p: float) -> ToyBlock:
    """Alg. 2 steps 3-4: same weights, attention replaced by SpargeAttn2(., ., ., k%, p%); the teacher is frozen."""
    student = copy.deepcopy(teacher)
    student.k_frac, student.top_p, student._full = float(k_frac), float(top_p), None
    for p in teacher.parameters():
        p.requires_grad_(False)
    return student


def noisy_latent(x1: torch.Tensor, x0: torch.Tensor, t: torch.Tensor) -> torch.Tensor:
    """x_t = t x_1 + (1 - t) x_0 (Alg. 2 step 7), t of shape [B]."""
    t = t.view(-1, *([1] * (x1.dim() - 1)))
    return t * x1 + (1.0 - t) * x0


class _VelocityDistillationLoss(torch.autograd.Function):
    """weight * ||u_sparse - u_full||^2 through the fused kernels: one pass for the loss, one for the gradient."""

    @staticmethod
    def forward(ctx, u_sparse, u_full, weight):
        u_full = u_full.detach()
        loss = torch.empty((), dtype=torch.float64, device=u_sparse.device)
        ws = torch.empty(_b.spa2_vd_loss_workspace_bytes(), dtype=torch.uint8, device=u_sparse.device)
        _b.spa2_vd_loss(u_sparse.detach(), u_full, weight, loss, ws)
        ctx.save_for_backward(u_sparse, u_full)
        ctx.weight = weight
        return loss

    @staticmethod
    def backward(ctx, upstream):
        u_sparse, u_full = ctx.saved_tensors
        grad = torch.empty_like(u_sparse)
        _b.spa2_vd_loss_grad(u_sparse.detach(), u_full, ctx.weight, upstream.contiguous(), grad)
        return grad, None, None


def velocity_distillation_loss(u_sparse: torch.Tensor, u_full: torch.Tensor, reduction: str = "mean") -> torch.Tensor:
    """L_VD = ||u_sparse - u_full||^2 (Sec. 4.2; Alg. 2), a float64 scalar.  `reduction`: "mean" divides by the
    number of elements; "batch" divides by the size of the leading dimension, which is the paper's expectation over
    training samples of the squared norm.  The teacher's prediction gets no gradient (it is frozen)."""
    if reduction == "mean":
        weight = 1.0 / u_sparse.numel()
    elif reduction == "batch":
        weight = 1.0 / u_sparse.shape[0]
    else:
        raise ValueError('reduction is "mean" or "batch"')
    if not u_sparse.is_cuda:
        raise ValueError("spa2 runs on the GPU only: predictions must be CUDA tensors")
    u_full = u_full.to(u_sparse.dtype)
    return _VelocityDistillationLoss.apply(u_sparse.contiguous(), u_full.contiguous(), weight)


def distill(student: torch.nn.Module, teacher: torch.nn.Module, batches: Iterable[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]],
            lr: float = 1e-3, on_step: Optional[Callable[[int, float], None]] = None) -> Dict[str, list]:
    """The loop of Alg. 2 over `batches` of (x_1, x_0, t): teacher and student see the same x_t, only the student
    is updated.  Returns the loss per step."""
    opt = torch.optim.Adam([p for p in student.parameters() if p.requires_grad], lr=lr)
    losses = []
    for step, (x1, x0, t) in enumerate(batches):
        xt = noisy_latent(x1, x0, t)
        with torch.no_grad():
            u_full = teacher(xt)
        loss = velocity_distillation_loss(student(xt), u_full)
        opt.zero_grad(set_to_none=True)
        loss.backward()
        opt.step()
        losses.append(float(loss.item()))
        if on_step is not None:
            on_step(step, losses[-1])
    return {"loss": losses}
