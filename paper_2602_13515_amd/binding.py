"""ctypes binding of libspa2.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/spa2.h)
and does nothing but turn torch tensors into device pointers, fill the two C
structs and raise on a negative return code.  All arithmetic runs in the HIP
kernels.  torch is used for device memory and the current stream, nothing else.
There is no CPU fallback: if the shared library is missing, importing any entry
point raises.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Optional

import torch  # must be imported before the library so that one HIP runtime (torch's) serves both

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libspa2.so")

BQ, BKV = 128, 64


class Spa2Error(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: spa2 error {code}: {spa2_strerror(code)}")


class _Shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("d", ctypes.c_int32),
                ("bq", ctypes.c_int32), ("bkv", ctypes.c_int32),
                ("sb", ctypes.c_int64), ("sh", ctypes.c_int64), ("sn", ctypes.c_int64)]


class _Pattern(ctypes.Structure):
    _fields_ = [("mask", ctypes.c_void_p), ("row_cnt", ctypes.c_void_p), ("row_idx", ctypes.c_void_p),
                ("col_cnt", ctypes.c_void_p), ("col_idx", ctypes.c_void_p),
                ("row_order", ctypes.c_void_p), ("col_order", ctypes.c_void_p)]


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2602_13515_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    shp, pat = ctypes.POINTER(_Shape), ctypes.POINTER(_Pattern)
    lib.spa2_version.restype = ctypes.c_int
    lib.spa2_version.argtypes = []
    lib.spa2_strerror.restype = ctypes.c_char_p
    lib.spa2_strerror.argtypes = [ctypes.c_int]
    lib.spa2_topk_blocks.restype = i32
    lib.spa2_topk_blocks.argtypes = [ctypes.c_double, i32]
    lib.spa2_mask_workspace_bytes.restype = sz
    lib.spa2_mask_workspace_bytes.argtypes = [shp]
    lib.spa2_bwd_workspace_bytes.restype = sz
    lib.spa2_bwd_workspace_bytes.argtypes = [shp]
    lib.spa2_bwd_workspace_min_bytes.restype = sz
    lib.spa2_bwd_workspace_min_bytes.argtypes = [shp]
    lib.spa2_fwd_workspace_bytes.restype = sz
    lib.spa2_fwd_workspace_bytes.argtypes = [shp]
    lib.spa2_mask.restype = ctypes.c_int
    lib.spa2_mask.argtypes = [vp, vp, shp, i32, f32, f32, pat, vp, vp, sz, vp]
    lib.spa2_pattern_full.restype = ctypes.c_int
    lib.spa2_pattern_full.argtypes = [shp, pat, vp]
    lib.spa2_fwd.restype = ctypes.c_int
    lib.spa2_fwd.argtypes = [vp, vp, vp, shp, pat, f32, vp, vp, vp, vp, sz, vp]
    lib.spa2_bwd.restype = ctypes.c_int
    lib.spa2_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, shp, pat, f32, vp, vp, vp, vp, sz, vp]
    lib.spa2_bwd_static.restype = ctypes.c_int
    lib.spa2_bwd_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, shp, pat, f32, vp, vp, vp, vp]
    lib.spa2_mask_pool.restype = ctypes.c_int
    lib.spa2_mask_pool.argtypes = [vp, vp, shp, vp, sz, vp]
    lib.spa2_mask_select.restype = ctypes.c_int
    lib.spa2_mask_select.argtypes = [shp, i32, f32, f32, pat, vp, vp, sz, vp]
    lib.spa2_mask_columns.restype = ctypes.c_int
    lib.spa2_mask_columns.argtypes = [shp, pat, vp]
    lib.spa2_bwd_delta.restype = ctypes.c_int
    lib.spa2_bwd_delta.argtypes = [vp, vp, vp, shp, vp, sz, vp]
    lib.spa2_bwd_dkdv.restype = ctypes.c_int
    lib.spa2_bwd_dkdv.argtypes = [vp, vp, vp, vp, vp, shp, pat, f32, vp, vp, vp, sz, vp]
    lib.spa2_bwd_dq.restype = ctypes.c_int
    lib.spa2_bwd_dq.argtypes = [vp, vp, vp, vp, vp, shp, pat, f32, vp, vp, sz, vp]
    lib.spa2_error_workspace_bytes.restype = sz
    lib.spa2_error_workspace_bytes.argtypes = [shp]
    lib.spa2_error_terms.restype = ctypes.c_int
    lib.spa2_error_terms.argtypes = [vp, vp, vp, vp, shp, vp, vp, sz, vp]
    lib.spa2_vd_loss_workspace_bytes.restype = sz
    lib.spa2_vd_loss_workspace_bytes.argtypes = []
    lib.spa2_vd_loss.restype = ctypes.c_int
    lib.spa2_vd_loss.argtypes = [vp, vp, ctypes.c_int64, i32, ctypes.c_double, vp, vp, sz, vp]
    lib.spa2_vd_loss_grad.restype = ctypes.c_int
    lib.spa2_vd_loss_grad.argtypes = [vp, vp, ctypes.c_int64, i32, ctypes.c_double, vp, vp, vp]
    _lib = lib
    return lib


EXPORTED_SYMBOLS = ("spa2_version", "spa2_strerror", "spa2_topk_blocks", "spa2_mask_workspace_bytes",
                    "spa2_bwd_workspace_bytes", "spa2_bwd_workspace_min_bytes", "spa2_fwd_workspace_bytes", "spa2_mask", "spa2_mask_pool", "spa2_mask_select",
                    "spa2_mask_columns", "spa2_pattern_full", "spa2_fwd", "spa2_bwd", "spa2_bwd_static", "spa2_bwd_delta",
                    "spa2_bwd_dkdv", "spa2_bwd_dq", "spa2_error_workspace_bytes", "spa2_error_terms",
                    "spa2_vd_loss_workspace_bytes", "spa2_vd_loss", "spa2_vd_loss_grad")


# ------------------------------------------------------------------ plumbing (memory only)
@dataclasses.dataclass
class Pattern:
    """Device buffers of a block-sparse pattern (spa2_pattern in the header)."""
    mask: torch.Tensor       # uint8 [B,H,Tm,Tn]
    row_cnt: torch.Tensor    # int32 [B,H,Tm]
    row_idx: torch.Tensor    # int32 [B,H,Tm,Tn]
    col_cnt: Optional[torch.Tensor]  # int32 [B,H,Tn]
    col_idx: Optional[torch.Tensor]  # int32 [B,H,Tn,Tm]
    row_order: Optional[torch.Tensor] = None  # int32 [B,H,Tm] launch order of query blocks (optional)
    col_order: Optional[torch.Tensor] = None  # int32 [B,H,Tn] launch order of key blocks (optional)

    def _c(self) -> _Pattern:
        return _Pattern(self.mask.data_ptr(), self.row_cnt.data_ptr(), self.row_idx.data_ptr(),
                        self.col_cnt.data_ptr() if self.col_cnt is not None else None,
                        self.col_idx.data_ptr() if self.col_idx is not None else None,
                        self.row_order.data_ptr() if self.row_order is not None else None,
                        self.col_order.data_ptr() if self.col_order is not None else None)


def alloc_pattern(B: int, H: int, N: int, device, columns: bool = True, col_order: bool = True) -> Pattern:
    Tm, Tn = -(-N // BQ), -(-N // BKV)
    i32 = torch.int32
    return Pattern(
        mask=torch.empty((B, H, Tm, Tn), dtype=torch.uint8, device=device),
        row_cnt=torch.empty((B, H, Tm), dtype=i32, device=device),
        row_idx=torch.empty((B, H, Tm, Tn), dtype=i32, device=device),
        col_cnt=torch.empty((B, H, Tn), dtype=i32, device=device) if columns else None,
        col_idx=torch.empty((B, H, Tn, Tm), dtype=i32, device=device) if columns else None,
        col_order=torch.empty((B, H, Tn), dtype=i32, device=device) if (columns and col_order) else None,
    )


def _shape_of(x: torch.Tensor) -> _Shape:
    if x.dim() != 4:
        raise ValueError("token tensors are 4-D views [B, H, N, d] (any batch/head/token strides, d contiguous)")
    if x.dtype != torch.bfloat16:
        raise ValueError("token tensors are bf16")
    if x.stride(3) != 1:
        raise ValueError("the head dimension must be contiguous")
    B, H, N, d = x.shape
    return _Shape(B, H, N, d, BQ, BKV, x.stride(0), x.stride(1), x.stride(2))


def _same_layout(ref: torch.Tensor, *others: torch.Tensor):
    for t in others:
        if t.shape != ref.shape or t.stride() != ref.stride() or t.dtype != ref.dtype or t.device != ref.device:
            raise ValueError("all token tensors of one call share shape, strides, dtype and device")


def _stream(x: torch.Tensor) -> int:
    return torch.cuda.current_stream(x.device).cuda_stream


def _check(rc: int, where: str):
    if rc != 0:
        raise Spa2Error(rc, where)


# ------------------------------------------------------------------ entry points
def spa2_version() -> int:
    return int(_load().spa2_version())


def spa2_strerror(code: int) -> str:
    return _load().spa2_strerror(int(code)).decode()


def spa2_topk_blocks(k_frac: float, Tn: int) -> int:
    return int(_load().spa2_topk_blocks(float(k_frac), int(Tn)))


def spa2_mask_workspace_bytes(q: torch.Tensor) -> int:
    return int(_load().spa2_mask_workspace_bytes(ctypes.byref(_shape_of(q))))


def spa2_bwd_workspace_bytes(q: torch.Tensor) -> int:
    return int(_load().spa2_bwd_workspace_bytes(ctypes.byref(_shape_of(q))))


def spa2_bwd_workspace_min_bytes(q: torch.Tensor) -> int:
    return int(_load().spa2_bwd_workspace_min_bytes(ctypes.byref(_shape_of(q))))


def spa2_fwd_workspace_bytes(q: torch.Tensor) -> int:
    return int(_load().spa2_fwd_workspace_bytes(ctypes.byref(_shape_of(q))))


def spa2_mask(q: torch.Tensor, k: torch.Tensor, topk_blocks: int, top_p: float, scale: float,
              out: Pattern, pbar_out: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    _same_layout(q, k)
    shape = _shape_of(q)
    pat = out._c()
    rc = _load().spa2_mask(q.data_ptr(), k.data_ptr(), ctypes.byref(shape), int(topk_blocks), float(top_p),
                           float(scale), ctypes.byref(pat),
                           pbar_out.data_ptr() if pbar_out is not None else None,
                           workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream(q))
    _check(rc, "spa2_mask")


def spa2_pattern_full(like: torch.Tensor, out: Pattern) -> None:
    shape = _shape_of(like)
    pat = out._c()
    _check(_load().spa2_pattern_full(ctypes.byref(shape), ctypes.byref(pat), _stream(like)), "spa2_pattern_full")


def spa2_fwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, pattern: Pattern, scale: float,
             o: torch.Tensor, lse: torch.Tensor, o_res: Optional[torch.Tensor] = None,
             workspace: Optional[torch.Tensor] = None) -> None:
    _same_layout(q, k, v, o, *([o_res] if o_res is not None else []))
    shape = _shape_of(q)
    pat = pattern._c()
    rc = _load().spa2_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), ctypes.byref(shape), ctypes.byref(pat),
                          float(scale), o.data_ptr(), o_res.data_ptr() if o_res is not None else None,
                          lse.data_ptr(), workspace.data_ptr() if workspace is not None else None,
                          _nbytes(workspace) if workspace is not None else 0, _stream(q))
    _check(rc, "spa2_fwd")


def spa2_bwd(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, o: torch.Tensor, d_o: torch.Tensor,
             lse: torch.Tensor, pattern: Pattern, scale: float, dq: torch.Tensor, dk: torch.Tensor,
             dv: torch.Tensor, workspace: torch.Tensor, o_res: Optional[torch.Tensor] = None) -> None:
    _same_layout(q, k, v, o, d_o, dq, dk, dv, *([o_res] if o_res is not None else []))
    shape = _shape_of(q)
    pat = pattern._c()
    rc = _load().spa2_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                          o_res.data_ptr() if o_res is not None else None, d_o.data_ptr(), lse.data_ptr(),
                          ctypes.byref(shape), ctypes.byref(pat), float(scale), dq.data_ptr(), dk.data_ptr(),
                          dv.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                          _stream(q))
    _check(rc, "spa2_bwd")


STATIC_MAX_ROWS = 4 * 1024 * 1024   # SPA2_STATIC_MAX_ROWS of the header


def spa2_bwd_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, o: torch.Tensor, d_o: torch.Tensor,
                    lse: torch.Tensor, pattern: Pattern, scale: float, dq: torch.Tensor, dk: torch.Tensor,
                    dv: torch.Tensor, o_res: Optional[torch.Tensor] = None) -> None:
    """spa2_bwd without a workspace: D lives in the library's fixed per-GPU array (B*H*N <= STATIC_MAX_ROWS)."""
    _same_layout(q, k, v, o, d_o, dq, dk, dv, *([o_res] if o_res is not None else []))
    shape = _shape_of(q)
    pat = pattern._c()
    with torch.cuda.device(q.device):      # the library looks its array up on the current device
        rc = _load().spa2_bwd_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                     o_res.data_ptr() if o_res is not None else None, d_o.data_ptr(),
                                     lse.data_ptr(), ctypes.byref(shape), ctypes.byref(pat), float(scale),
                                     dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), _stream(q))
    _check(rc, "spa2_bwd_static")


# ------------------------------------------------------------------ the stages of spa2_mask / spa2_bwd, one by one
def _nbytes(t: torch.Tensor) -> int:
    return t.numel() * t.element_size()


def spa2_mask_pool(q: torch.Tensor, k: torch.Tensor, workspace: torch.Tensor) -> None:
    _same_layout(q, k)
    shape = _shape_of(q)
    _check(_load().spa2_mask_pool(q.data_ptr(), k.data_ptr(), ctypes.byref(shape), workspace.data_ptr(),
                                  _nbytes(workspace), _stream(q)), "spa2_mask_pool")


def spa2_mask_select(like: torch.Tensor, topk_blocks: int, top_p: float, scale: float, out: Pattern,
                     pbar_out: Optional[torch.Tensor], workspace: torch.Tensor) -> None:
    shape = _shape_of(like)
    pat = out._c()
    _check(_load().spa2_mask_select(ctypes.byref(shape), int(topk_blocks), float(top_p), float(scale),
                                    ctypes.byref(pat), pbar_out.data_ptr() if pbar_out is not None else None,
                                    workspace.data_ptr(), _nbytes(workspace), _stream(like)), "spa2_mask_select")


def spa2_mask_columns(like: torch.Tensor, out: Pattern) -> None:
    shape = _shape_of(like)
    pat = out._c()
    _check(_load().spa2_mask_columns(ctypes.byref(shape), ctypes.byref(pat), _stream(like)), "spa2_mask_columns")


def spa2_bwd_delta(o: torch.Tensor, d_o: torch.Tensor, workspace: torch.Tensor,
                   o_res: Optional[torch.Tensor] = None) -> None:
    _same_layout(o, d_o, *([o_res] if o_res is not None else []))
    shape = _shape_of(o)
    _check(_load().spa2_bwd_delta(o.data_ptr(), o_res.data_ptr() if o_res is not None else None, d_o.data_ptr(),
                                  ctypes.byref(shape), workspace.data_ptr(),
                                  _nbytes(workspace), _stream(o)), "spa2_bwd_delta")


def spa2_bwd_dkdv(q, k, v, d_o, lse, pattern: Pattern, scale: float, dk, dv, workspace) -> None:
    _same_layout(q, k, v, d_o, dk, dv)
    shape = _shape_of(q)
    pat = pattern._c()
    _check(_load().spa2_bwd_dkdv(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(), lse.data_ptr(),
                                 ctypes.byref(shape), ctypes.byref(pat), float(scale), dk.data_ptr(), dv.data_ptr(),
                                 workspace.data_ptr(), _nbytes(workspace), _stream(q)), "spa2_bwd_dkdv")


def spa2_bwd_dq(q, k, v, d_o, lse, pattern: Pattern, scale: float, dq, workspace) -> None:
    _same_layout(q, k, v, d_o, dq)
    shape = _shape_of(q)
    pat = pattern._c()
    _check(_load().spa2_bwd_dq(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(), lse.data_ptr(),
                               ctypes.byref(shape), ctypes.byref(pat), float(scale), dq.data_ptr(),
                               workspace.data_ptr(), _nbytes(workspace), _stream(q)), "spa2_bwd_dq")


# ------------------------------------------------------------------ diagnostics
def spa2_error_workspace_bytes(o: torch.Tensor) -> int:
    return int(_load().spa2_error_workspace_bytes(ctypes.byref(_shape_of(o))))


def spa2_error_terms(o_sparse: torch.Tensor, o_dense: torch.Tensor, lse_sparse: torch.Tensor,
                     lse_dense: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor) -> None:
    """out: float64 [B, H, 5] = sums of |o_dense - o_sparse|, |o_dense|, |dropped|, |renormalisation|, tau."""
    _same_layout(o_sparse, o_dense)
    if out.dtype != torch.float64 or not out.is_contiguous():
        raise ValueError("out is a contiguous float64 [B, H, 5] tensor")
    rc = _load().spa2_error_terms(o_sparse.data_ptr(), o_dense.data_ptr(), lse_sparse.data_ptr(),
                                  lse_dense.data_ptr(), ctypes.byref(_shape_of(o_sparse)), out.data_ptr(),
                                  workspace.data_ptr(), _nbytes(workspace), _stream(o_sparse))
    _check(rc, "spa2_error_terms")


_VD_DTYPES = {torch.bfloat16: 0, torch.float32: 1}


def _vd_args(u_sparse: torch.Tensor, u_full: torch.Tensor):
    if not (u_sparse.is_cuda and u_full.is_cuda):
        raise ValueError("spa2 runs on the GPU only: predictions must be CUDA tensors")
    if u_sparse.dtype not in _VD_DTYPES or u_full.dtype != u_sparse.dtype:
        raise ValueError("predictions are bfloat16 or float32, both of the same type")
    if u_sparse.shape != u_full.shape or not u_sparse.is_contiguous() or not u_full.is_contiguous():
        raise ValueError("predictions are contiguous tensors of one shape")
    return u_sparse.numel(), _VD_DTYPES[u_sparse.dtype]


def spa2_vd_loss_workspace_bytes() -> int:
    return int(_load().spa2_vd_loss_workspace_bytes())


def spa2_vd_loss(u_sparse: torch.Tensor, u_full: torch.Tensor, weight: float, loss: torch.Tensor,
                 workspace: torch.Tensor) -> None:
    """loss (float64, one element) = weight * sum (u_sparse - u_full)^2."""
    n, dt = _vd_args(u_sparse, u_full)
    if loss.dtype != torch.float64 or loss.numel() != 1:
        raise ValueError("loss is a float64 tensor of one element")
    _check(_load().spa2_vd_loss(u_sparse.data_ptr(), u_full.data_ptr(), n, dt, float(weight), loss.data_ptr(),
                                workspace.data_ptr(), _nbytes(workspace), _stream(u_sparse)), "spa2_vd_loss")


def spa2_vd_loss_grad(u_sparse: torch.Tensor, u_full: torch.Tensor, weight: float, upstream: Optional[torch.Tensor],
                      grad: torch.Tensor) -> None:
    """grad = upstream * 2 * weight * (u_sparse - u_full); upstream is a float64 device scalar or None (= 1)."""
    n, dt = _vd_args(u_sparse, u_full)
    if grad.dtype != u_sparse.dtype or grad.shape != u_sparse.shape or not grad.is_contiguous():
        raise ValueError("grad has the type and shape of the predictions and is contiguous")
    if upstream is not None and (upstream.dtype != torch.float64 or upstream.numel() != 1 or not upstream.is_cuda):
        raise ValueError("upstream is a float64 CUDA tensor of one element")
    _check(_load().spa2_vd_loss_grad(u_sparse.data_ptr(), u_full.data_ptr(), n, dt, float(weight),
                                     None if upstream is None else upstream.data_ptr(), grad.data_ptr(),
                                     _stream(u_sparse)), "spa2_vd_loss_grad")
