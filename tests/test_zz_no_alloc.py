"""spa2_bwd_static (the backward pass for callers that cannot allocate: D lives in the library's fixed
per-GPU array) against spa2_bwd with a caller's workspace: same kernels, so the gradients must be
identical bit for bit.  Two calls in a row, the second on a smaller input, so that the second call
runs over what the first one left in the array."""
import math

import pytest
import torch

import paper_2602_13515_amd as spa2
from paper_2602_13515_amd import workloads as wl

from gpu_util import dev, gpu_bwd, gpu_fwd, gpu_mask

pytestmark = pytest.mark.gpu


def _both_ways(w, seed):
    q, k, v, do = wl.make_inputs(w, seed=seed, device=dev())
    scale = 1.0 / math.sqrt(w.d)
    pat, _ = gpu_mask(q, k, spa2.spa2_topk_blocks(w.k_frac, w.Tn), w.top_p, want_pbar=False)
    o, lse, o_res = gpu_fwd(q, k, v, pat, residual=True)
    # (the mandatory part of the workspace only, as the static path has: no list is split on either side)
    ref = gpu_bwd(q, k, v, o, do, lse, pat, o_res=o_res, split=False)
    got = tuple(torch.full_like(q, float("nan")) for _ in range(3))
    spa2.spa2_bwd_static(q, k, v, o, do, lse, pat, scale, *got, o_res=o_res)
    torch.cuda.synchronize()
    for name, g, r in zip(("dQ", "dK", "dV"), got, ref):
        assert torch.isfinite(g).all(), name
        assert torch.equal(g, r), f"{name}: spa2_bwd_static differs from spa2_bwd on {w.name}"


def test_static_backward_equals_workspace_backward_twice():
    big = wl.Workload("static-a", 2, 3, 3000, 128, 0.2, 0.7, "lowrank", True)
    small = wl.Workload("static-b", 1, 2, 777, 64, 0.3, 0.6, "gaussian", True)
    print(f"call 1: {big.name} B={big.B} H={big.H} N={big.N} d={big.d}", flush=True)
    _both_ways(big, seed=11)
    print(f"call 2: {small.name} B={small.B} H={small.H} N={small.N} d={small.d}", flush=True)
    _both_ways(small, seed=12)


def test_static_backward_rejects_sizes_beyond_its_array():
    """B*H*N above SPA2_STATIC_MAX_ROWS: error before any launch, outputs untouched (checked on the host:
    the shape is only described, no tensor of that size exists)."""
    from paper_2602_13515_amd import binding
    import ctypes
    lib = binding._load()
    N = binding.STATIC_MAX_ROWS // 4 + 64
    shape = binding._Shape(1, 4, N, 128, 128, 64, 4 * N * 128, N * 128, 128)
    fake = ctypes.c_void_p(0x1000)
    full = binding._Pattern(0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    rc = lib.spa2_bwd_static(fake, fake, fake, fake, None, fake, fake, ctypes.byref(shape), ctypes.byref(full),
                             0.1, fake, fake, fake, None)
    assert rc == -6, rc
