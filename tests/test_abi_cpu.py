"""Host-side checks that need no GPU: the shared library loads, exports every symbol the
header declares, validates its arguments before any launch, and the k% -> block-count rule
agrees with the oracle's."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import spa2_oracle as orc
from paper_2602_13515_amd import binding
from paper_2602_13515_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "spa2.h")


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spa2_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding._load()
    names = _declared()
    assert set(names) == set(binding.EXPORTED_SYMBOLS), names
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_error_strings():
    assert binding.spa2_version() >= 100
    seen = set()
    for code in range(0, -8, -1):
        s = binding.spa2_strerror(code)
        assert s and s not in seen
        seen.add(s)
    assert "unknown" in binding.spa2_strerror(-99)


def test_topk_blocks_matches_oracle_rule():
    for tn in (1, 2, 7, 10, 32, 512, 1182, 4096):
        for k in (0.0, 1e-9, 0.01, 0.03, 0.05, 0.1, 0.2, 0.25, 0.5, 0.999, 1.0, 2.0):
            assert binding.spa2_topk_blocks(k, tn) == orc.topk_blocks(k, tn), (k, tn)
    assert binding.spa2_topk_blocks(0.2, 10) == 2          # Case 1 of Sec. 3.2
    assert binding.spa2_topk_blocks(0.05, 1182) == 60


def _shape(B=1, H=2, N=300, d=128, bq=128, bkv=64, sb=None, sh=None, sn=None):
    sn = d if sn is None else sn
    sh = N * sn if sh is None else sh
    sb = H * sh if sb is None else sb
    return binding._Shape(B, H, N, d, bq, bkv, sb, sh, sn)


def test_argument_validation_happens_on_the_host():
    """Every rejected call returns before touching the device (there is none here)."""
    lib = binding._load()
    pat = binding._Pattern(None, None, None, None, None)
    fake = ctypes.c_void_p(0x1000)           # 16-byte aligned, never dereferenced on these paths
    odd = ctypes.c_void_p(0x1004)
    ok = _shape()
    f = lib.spa2_fwd
    assert f(None, fake, fake, ctypes.byref(ok), ctypes.byref(pat), 0.1, fake, None, fake, None, 0, None) == -1
    assert f(fake, fake, fake, None, ctypes.byref(pat), 0.1, fake, None, fake, None, 0, None) == -1
    assert f(fake, fake, fake, ctypes.byref(ok), ctypes.byref(pat), 0.1, fake, None, fake, None, 0, None) == -1   # empty pattern
    full = binding._Pattern(0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    assert f(odd, fake, fake, ctypes.byref(ok), ctypes.byref(full), 0.1, fake, None, fake, None, 0, None) == -4
    assert f(fake, fake, fake, ctypes.byref(ok), ctypes.byref(full), 0.0, fake, None, fake, None, 0, None) == -5
    assert f(fake, fake, fake, ctypes.byref(_shape(d=96)), ctypes.byref(full), 0.1, fake, None, fake, None, 0, None) == -3
    assert f(fake, fake, fake, ctypes.byref(_shape(bq=64)), ctypes.byref(full), 0.1, fake, None, fake, None, 0, None) == -3
    assert f(fake, fake, fake, ctypes.byref(_shape(N=0)), ctypes.byref(full), 0.1, fake, None, fake, None, 0, None) == -2
    assert f(fake, fake, fake, ctypes.byref(_shape(sn=132)), ctypes.byref(full), 0.1, fake, None, fake, None, 0, None) == -4
    wide = _shape(sn=(1 << 23) + 8, sh=1 << 40, sb=1 << 41)       # a tile's rows would not fit a 32-bit offset
    assert f(fake, fake, fake, ctypes.byref(wide), ctypes.byref(full), 0.1, fake, None, fake, None, 0, None) == -2
    m = lib.spa2_mask
    big = 1 << 30
    assert m(fake, fake, ctypes.byref(ok), 1, 0.5, 0.1, ctypes.byref(full), None, None, big, None) == -6
    assert m(fake, fake, ctypes.byref(ok), 1, 0.5, 0.1, ctypes.byref(full), None, fake, 16, None) == -6
    assert m(fake, fake, ctypes.byref(ok), 0, 0.0, 0.1, ctypes.byref(full), None, fake, big, None) == -5
    assert m(fake, fake, ctypes.byref(ok), 6, 0.5, 0.1, ctypes.byref(full), None, fake, big, None) == -5   # Tn = 5
    assert m(fake, fake, ctypes.byref(ok), 1, 1.5, 0.1, ctypes.byref(full), None, fake, big, None) == -5
    assert m(fake, fake, ctypes.byref(ok), 1, float("nan"), 0.1, ctypes.byref(full), None, fake, big, None) == -5
    assert m(fake, fake, ctypes.byref(_shape(N=64 * 8193, d=64)), 1, 0.5, 0.1, ctypes.byref(full), None, fake,
             1 << 40, None) == -2                                                                      # row too long
    # spa2_mask_columns alone refuses rows longer than its sort holds (N > 524,288), like spa2_mask does
    assert lib.spa2_mask_columns(ctypes.byref(_shape(N=64 * 8193, d=64)), ctypes.byref(full), None) == -2
    # B*H*(T_m + T_n) workgroups must fit a 32-bit grid: 2^24 heads of 20,000 tokens do not
    many = _shape(B=1 << 12, H=1 << 12, N=20000, d=64)
    assert lib.spa2_mask_columns(ctypes.byref(many), ctypes.byref(full), None) == -2
    assert f(fake, fake, fake, ctypes.byref(many), ctypes.byref(full), 0.1, fake, None, fake, None, 0, None) == -2
    # the workspace-free backward: same checks, and its fixed array bounds B*H*N
    bs = lib.spa2_bwd_static
    sargs = [fake, fake, fake, fake, None, fake, fake]
    assert bs(*sargs, None, ctypes.byref(full), 0.1, fake, fake, fake, None) == -1
    too_long = _shape(B=1, H=4, N=binding.STATIC_MAX_ROWS // 4 + 64, d=128)
    assert bs(*sargs, ctypes.byref(too_long), ctypes.byref(full), 0.1, fake, fake, fake, None) == -6
    half = binding._Pattern(0x1000, 0x1000, 0x1000, 0x1000, None)
    assert m(fake, fake, ctypes.byref(ok), 1, 0.5, 0.1, ctypes.byref(half), None, fake, big, None) == -1
    b = lib.spa2_bwd
    norows = binding._Pattern(0x1000, 0x1000, 0x1000, None, None)
    args = [fake, fake, fake, fake, None, fake, fake]
    assert b(*args, ctypes.byref(ok), ctypes.byref(norows), 0.1, fake, fake, fake, fake, big, None) == -1
    assert b(*args, ctypes.byref(ok), ctypes.byref(full), 0.1, fake, fake, fake, fake, 8, None) == -6
    assert lib.spa2_pattern_full(ctypes.byref(ok), None, None) == -1
    vd, vg = lib.spa2_vd_loss, lib.spa2_vd_loss_grad
    assert vd(None, fake, 8, 0, 1.0, fake, fake, big, None) == -1
    assert vd(fake, fake, 0, 0, 1.0, fake, fake, big, None) == -2
    assert vd(fake, fake, 8, 2, 1.0, fake, fake, big, None) == -3            # element type
    assert vd(odd, fake, 8, 1, 1.0, fake, fake, big, None) == -4
    assert vd(fake, fake, 8, 1, 0.0, fake, fake, big, None) == -5
    assert vd(fake, fake, 8, 1, float("inf"), fake, fake, big, None) == -5
    assert vd(fake, fake, 8, 1, 1.0, fake, fake, 64, None) == -6
    assert vd(fake, fake, 8, 1, 1.0, None, fake, big, None) == -1
    assert vg(fake, fake, 8, 1, 1.0, None, None, None) == -1
    assert vg(fake, fake, 8, 1, 1.0, None, odd, None) == -4
    assert lib.spa2_vd_loss_workspace_bytes() >= 2048 * 8


def test_workspace_sizes():
    lib = binding._load()
    s = _shape(B=2, H=3, N=1000, d=128)
    tm, tn = 8, 16
    need = lib.spa2_mask_workspace_bytes(ctypes.byref(s))
    assert need >= 6 * (tm + tn) * 128 * 4 and need % 256 == 0
    assert lib.spa2_bwd_workspace_bytes(ctypes.byref(s)) >= 6 * 1000 * 4
    assert lib.spa2_mask_workspace_bytes(ctypes.byref(_shape(d=100))) == 0


def test_binding_rejects_bad_tensors_before_calling_c():
    import torch
    q = torch.zeros((1, 1, 128, 128), dtype=torch.float32)
    with pytest.raises(ValueError):
        binding._shape_of(q)
    with pytest.raises(ValueError):
        binding._shape_of(torch.zeros((1, 128, 128), dtype=torch.bfloat16))
    with pytest.raises(ValueError):
        binding._shape_of(torch.zeros((1, 1, 128, 128), dtype=torch.bfloat16).transpose(2, 3))


# ------------------------------------------------------------------ workload generators
def test_workload_shapes_and_determinism():
    assert (wl.WAN13_95.Tm, wl.WAN13_95.Tn) == (256, 512)
    assert (wl.WAN14_95.Tm, wl.WAN14_95.Tn) == (591, 1182)
    assert (wl.TINY.Tm, wl.TINY.Tn) == (16, 32)
    a = wl.make_inputs(wl.TINY, seed=0)
    b = wl.make_inputs(wl.TINY, seed=0)
    c = wl.make_inputs(wl.TINY, seed=1)
    import torch
    for x, y in zip(a, b):
        assert x.dtype == torch.bfloat16 and x.shape == (1, 2, 2048, 64)
        assert torch.equal(x, y)
    assert not torch.equal(a[0], c[0])
    # one head regenerated alone equals the same head of the full draw
    qh, kh, vh, doh = wl.head_inputs(wl.TINY, 0, 1, seed=0)
    assert torch.equal(qh, a[0][0, 1]) and torch.equal(doh, a[3][0, 1])


def test_lowrank_recipe_gives_skewed_pooled_rows_and_target_sparsity():
    w = wl.Workload("probe", 1, 1, 8192, 128, 0.05, 0.8, "lowrank", False)
    q, k, _, _ = wl.head_inputs(w, 0, 0, seed=0, need_do=False)
    qd, kd = q.double().numpy(), k.double().numpy()
    sbar = orc.pool(qd, 128) @ orc.pool(kd, 64).T / np.sqrt(128)
    assert 4.5 < sbar.std() < 7.0                       # pooled logit = 4 * <a_q, a_k>, std about 5.7
    mask, _ = orc.block_mask(qd, kd, orc.topk_blocks(0.05, w.Tn), 0.8)
    assert 0.90 < 1.0 - mask.mean() < 0.95
    # pure Gaussian inputs pool to nearly uniform rows instead
    g = wl.Workload("g", 1, 1, 8192, 128, 0.05, 0.8, "gaussian", False)
    q, k, _, _ = wl.head_inputs(g, 0, 0, need_do=False)
    sb = orc.pool(q.double().numpy(), 128) @ orc.pool(k.double().numpy(), 64).T / np.sqrt(128)
    assert sb.std() < 0.05


def test_stress_recipe_has_uniform_and_sink_rows():
    w = wl.Workload("probe", 1, 1, 4096, 128, 0.05, 0.8, "stress", False)
    q, k, _, _ = wl.head_inputs(w, 0, 0, need_do=False)
    pbar = orc.pooled_map(q.double().numpy(), k.double().numpy())
    even, odd = pbar[0::2], pbar[1::2]
    assert np.abs(even * w.Tn - 1).max() < 0.02         # near-uniform rows
    assert (odd[:, 0] > 0.5).all()                      # the sink block dominates


def test_operator_has_no_cpu_path():
    import torch
    import paper_2602_13515_amd as spa2
    x = torch.zeros((1, 1, 128, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        spa2.sparge_attn2(x, x, x, 0.1, 0.5)
    with pytest.raises(ValueError):
        spa2.sparge_attn2(x.float(), x.float(), x.float(), 0.1, 0.5)


def test_header_is_plain_c():
    """The boundary is a C ABI: the header must compile as C99 without a HIP or C++ toolchain."""
    import shutil
    import subprocess
    import tempfile
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    with tempfile.TemporaryDirectory() as td:
        src = os.path.join(td, "t.c")
        with open(src, "w") as f:
            f.write('#include "spa2.h"\nint main(void) { spa2_shape s; spa2_pattern p; (void)s; (void)p; return SPA2_OK; }\n')
        r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                            "-I", os.path.join(ROOT, "include"), src], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_argument_checks_under_host_sanitizers():
    """The argument-check layer (csrc/api.hip) compiled with AddressSanitizer and UndefinedBehaviorSanitizer on the
    host side, linked against launcher stubs that abort, and driven by tests/abi_sanitize/driver.c with every kind
    of rejected call: no sanitizer report, no launcher reached, every error code as documented."""
    import shutil
    import subprocess
    import tempfile
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    clang = "/opt/rocm/lib/llvm/bin/clang"
    if not (os.path.exists(hipcc) and os.path.exists(clang)):
        pytest.skip("no ROCm toolchain")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2602_13515_amd", "csrc")]
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
    xsan = [x for s in san for x in ("-Xarch_host", s)]
    dev = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Wno-unused-command-line-argument",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    here = os.path.join(ROOT, "tests", "abi_sanitize")
    with tempfile.TemporaryDirectory() as td:
        o = lambda n: os.path.join(td, n)
        steps = [
            [clang, "-std=c99", "-g", "-c", *san, *inc, os.path.join(here, "driver.c"), "-o", o("driver.o")],
            [hipcc, *dev, *xsan, *inc, "-c", os.path.join(ROOT, "paper_2602_13515_amd", "csrc", "api.hip"), "-o", o("api.o")],
            [hipcc, *dev, *xsan, *inc, "-x", "hip", "-c", os.path.join(here, "launch_stubs.cpp"), "-o", o("stubs.o")],
        [hipcc, *dev, *xsan, *inc, "-c", os.path.join(ROOT, "paper_2602_13515_amd", "csrc", "split.hip"), "-o", o("split.o")],
            [hipcc, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
             o("api.o"), o("stubs.o"), o("split.o"), o("driver.o"), "-o", o("abi_check")],
        ]
        for cmd in steps:
            r = subprocess.run(cmd, capture_output=True, text=True)
            assert r.returncode == 0, r.stderr[-3000:]
        r = subprocess.run([o("abi_check")], capture_output=True, text=True, timeout=120)
        assert r.returncode == 0 and "all rejected before launch" in r.stdout, (r.stdout[-2000:], r.stderr[-3000:])
        assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-3000:]
