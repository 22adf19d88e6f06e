"""Seeded synthetic inputs shaped like the paper's video-DiT attention layers.

This module holds input recipes only: no pooling, masking or attention
arithmetic lives here, so both the GPU library's tests and the CPU checker can
draw the very same bf16 bits from it.  It imports neither of them.

The paper evaluates on Wan2.1-1.3B at 480p and Wan2.1-14B at 720p (Sec. 5.1),
whose real activations need the model weights; these generators stand in for
them with the same token counts, head counts and head dimension:

* ``gaussian``: Q, K, V, dO ~ N(0, 1) i.i.d.
* ``lowrank``:  per head a shared rank-4 component is added to Q and K,
  ``Q = G_q + 2 * a_q(n) U`` and ``K = G_k + 2 * a_k(n) U`` with U four
  orthonormal rows scaled by d**0.25 and a_q, a_k ~ N(0, 1) coefficient tables
  that are constant over 64-token chunks.  Block-coherent coefficients survive
  mean pooling, so the pooled map has realistic row skew (pure Gaussian Q, K
  pool to almost zero and every row would look uniform).
* ``stress``:   per head, even query blocks are scaled by 0.05 (near-uniform
  pooled rows: thousands of near-ties) and odd query blocks plus the first 64
  keys receive a shared direction with beta**2 / sqrt(d) = 6 (a sink block).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Iterable, Optional

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    N: int
    d: int
    k_frac: float
    top_p: float
    kind: str           # "gaussian" | "lowrank" | "stress"
    backward: bool

    @property
    def Tm(self) -> int:
        return -(-self.N // 128)

    @property
    def Tn(self) -> int:
        return -(-self.N // 64)


# The five configurations named by the benchmark definition.
TINY = Workload("tiny", 1, 2, 2048, 64, 0.25, 0.9, "gaussian", True)
WAN13_FWD = Workload("wan1.3b-480p-fwd", 1, 12, 32760, 128, 0.10, 0.9, "lowrank", False)
WAN13_95 = Workload("wan1.3b-480p-95", 1, 12, 32760, 128, 0.05, 0.8, "lowrank", True)
WAN14_95 = Workload("wan14b-720p-95", 1, 40, 75600, 128, 0.05, 0.8, "lowrank", True)
MASK_STRESS = Workload("mask-stress", 2, 12, 32768, 128, 0.05, 0.8, "stress", True)

CONFIGS = {w.name: w for w in (TINY, WAN13_FWD, WAN13_95, WAN14_95, MASK_STRESS)}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, g: torch.Generator, device) -> torch.Tensor:
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def head_inputs(w: Workload, b: int, h: int, seed: int = 0, device="cpu",
                need_do: bool = True):
    """bf16 (q, k, v, do) of shape [N, d] for one (batch, head).  The stream is
    seeded by (seed, b, h) alone, so any subset of heads can be regenerated
    independently, on either device type (CPU and GPU generators give
    different but equally valid draws; a parity test moves one draw to both
    sides)."""
    g = _gen(device, seed * 1_000_003 + (b * w.H + h) * 7919 + 17)
    N, d = w.N, w.d
    q = _randn((N, d), g, device)
    k = _randn((N, d), g, device)
    v = _randn((N, d), g, device)
    do = _randn((N, d), g, device) if need_do else None
    if w.kind == "lowrank":
        rank, chunk = 4, 64
        # the small basis is always drawn and orthonormalised on the CPU (no device linear algebra needed)
        gc = _gen("cpu", seed * 1_000_003 + (b * w.H + h) * 7919 + 18)
        basis, _ = torch.linalg.qr(_randn((d, rank), gc, "cpu"))       # [d, rank], orthonormal columns
        u = (basis.T.contiguous() * (d ** 0.25)).to(device)             # [rank, d]
        n_chunks = -(-N // chunk)
        cq = _randn((n_chunks, rank), g, device)
        ck = _randn((n_chunks, rank), g, device)
        tok = torch.arange(N, device=device) // chunk
        q = q + 2.0 * (cq[tok] @ u)
        k = k + 2.0 * (ck[tok] @ u)
    elif w.kind == "stress":
        wdir = _randn((d,), g, device)
        wdir = wdir / wdir.norm()
        beta = math.sqrt(6.0 * math.sqrt(d))
        qblk = torch.arange(N, device=device) // 128
        even = (qblk % 2 == 0)
        q = torch.where(even[:, None], q * 0.05, q + beta * wdir[None, :])
        k[:64] = k[:64] + beta * wdir[None, :]
    elif w.kind != "gaussian":
        raise ValueError(f"unknown workload kind {w.kind!r}")
    bf = torch.bfloat16
    return q.to(bf), k.to(bf), v.to(bf), (do.to(bf) if need_do else None)


def make_inputs(w: Workload, seed: int = 0, device="cpu", need_do: Optional[bool] = None,
                heads: Optional[Iterable[tuple]] = None):
    """bf16 tensors q, k, v, do of shape [B, H, N, d] (contiguous).  With
    ``heads`` (an iterable of (b, h)) only those heads are filled; the rest are
    left zero, which keeps large configurations cheap to sample."""
    if need_do is None:
        need_do = w.backward
    shape = (w.B, w.H, w.N, w.d)
    q = torch.zeros(shape, dtype=torch.bfloat16, device=device)
    k = torch.zeros_like(q)
    v = torch.zeros_like(q)
    do = torch.zeros_like(q) if need_do else None
    todo = list(heads) if heads is not None else [(b, h) for b in range(w.B) for h in range(w.H)]
    for (b, h) in todo:
        qh, kh, vh, doh = head_inputs(w, b, h, seed, device, need_do)
        q[b, h], k[b, h], v[b, h] = qh, kh, vh
        if need_do:
            do[b, h] = doh
    return q, k, v, do
