"""spa2: SpargeAttention2's hot path (hybrid Top-k+Top-p block masker, block-sparse
attention forward and backward) as hand-written HIP kernels for AMD MI355X (gfx950).

`binding` exposes the C ABI of libspa2.so one-to-one; `autograd` wraps the three calls into a
differentiable operator; `diagnostics` measures masking error and calibrates k% / p%; `distill` is the velocity
distillation step with its fused loss; `workloads` holds the seeded
synthetic input recipes; `build` compiles the library in-tree with hipcc.
"""
from .binding import (  # noqa: F401
    BKV, BQ, Pattern, Spa2Error, alloc_pattern, spa2_bwd, spa2_bwd_static, spa2_bwd_workspace_bytes, spa2_bwd_workspace_min_bytes, spa2_fwd_workspace_bytes, spa2_fwd, spa2_mask,
    spa2_mask_workspace_bytes, spa2_pattern_full, spa2_mask_pool, spa2_mask_select, spa2_mask_columns,
    spa2_bwd_delta, spa2_bwd_dkdv, spa2_bwd_dq, spa2_error_terms, spa2_error_workspace_bytes, spa2_strerror,
    spa2_topk_blocks, spa2_version, spa2_vd_loss, spa2_vd_loss_grad, spa2_vd_loss_workspace_bytes,
)
from .autograd import SpargeAttn2, build_pattern, sparge_attn2  # noqa: F401,E402
from .diagnostics import block_sparsity, calibrate, masking_error  # noqa: F401,E402
