"""Velocity distillation (Sec. 4.2, Alg. 2) on a toy block: the loss that compares the sparse student with its
full-attention teacher goes down when the student is trained through the block-sparse backward kernels."""
import pytest
import torch

from paper_2602_13515_amd import distill as vd

from gpu_util import dev

pytestmark = pytest.mark.gpu


def test_student_approaches_teacher():
    torch.manual_seed(0)
    B, N, dim, heads = 2, 1536, 128, 2
    teacher = vd.ToyBlock(dim, heads).to(dev())
    with torch.no_grad():                                   # sharper attention than the default initialisation gives
        teacher.qkv.weight.mul_(6.0)
    student = vd.make_student(teacher, k_frac=0.1, top_p=0.3)
    assert all(not p.requires_grad for p in teacher.parameters())
    g = torch.Generator(device=dev()).manual_seed(1)
    # one fixed pool of (x_1, x_0, t) triples, visited several times
    pool = [(torch.randn((B, N, dim), generator=g, device=dev()), torch.randn((B, N, dim), generator=g, device=dev()),
             torch.rand((B,), generator=g, device=dev())) for _ in range(4)]
    with torch.no_grad():
        before = sum(float(vd.velocity_distillation_loss(student(vd.noisy_latent(*b)), teacher(vd.noisy_latent(*b)))) for b in pool) / len(pool)
    hist = vd.distill(student, teacher, (pool[s % len(pool)] for s in range(40)), lr=2e-3)
    with torch.no_grad():
        after = sum(float(vd.velocity_distillation_loss(student(vd.noisy_latent(*b)), teacher(vd.noisy_latent(*b)))) for b in pool) / len(pool)
    print(f"L_VD before {before:.5f} after {after:.5f}; first/last step {hist['loss'][0]:.5f} {hist['loss'][-1]:.5f}", flush=True)
    assert before > 0 and all(l == l for l in hist["loss"])            # finite
    assert after < 0.8 * before
    for p in student.parameters():
        assert torch.isfinite(p).all()


def _predictions(n, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    u_f = torch.randn(n, generator=g).to(dtype)
    u_s = (u_f.float() + 0.1 * torch.randn(n, generator=g)).to(dtype)
    return u_s, u_f


# sizes: one element; less than one 16-byte vector; exactly one; a ragged tail; more vectors than the largest grid
# takes in one sweep (2048 workgroups x 256 lanes), again with a tail
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32], ids=["bf16", "f32"])
@pytest.mark.parametrize("n", [1, 7, 8, 1003, 5_000_003])
def test_fused_loss_and_gradient_match_the_oracle(n, dtype):
    import numpy as np
    from oracle import spa2_oracle as orc
    import paper_2602_13515_amd as spa2
    print(f"case n={n} dtype={dtype}", flush=True)
    u_s, u_f = _predictions(n, dtype, seed=n)
    weight = 1.0 / 3.0
    ref_loss, ref_grad = orc.vd_loss(u_s.double().numpy(), u_f.double().numpy(), weight)
    ds, df = u_s.to(dev()), u_f.to(dev())
    loss = torch.full((1,), -1.0, dtype=torch.float64, device=dev())
    ws = torch.empty(spa2.spa2_vd_loss_workspace_bytes(), dtype=torch.uint8, device=dev())
    spa2.spa2_vd_loss(ds, df, weight, loss, ws)
    # differences in fp32 (exact for bf16 inputs, 2^-24 relative for fp32), squares and sums in fp64
    assert abs(loss.item() - ref_loss) <= 1e-6 * ref_loss + 1e-300
    again = torch.zeros_like(loss)
    spa2.spa2_vd_loss(ds, df, weight, again, ws)
    assert again.item() == loss.item()                                   # fixed summation order
    for up in (None, torch.tensor([-2.5], dtype=torch.float64, device=dev())):
        grad = torch.full_like(ds, float("nan"))
        spa2.spa2_vd_loss_grad(ds, df, weight, up, grad)
        want = ref_grad * (1.0 if up is None else -2.5)
        got = grad.double().cpu().numpy()
        # one rounding of the product to the output type
        tol = (2.0 ** -8 if dtype == torch.bfloat16 else 2.0 ** -22) * np.abs(want) + 1e-30
        assert (np.abs(got - want) <= tol).all()


def test_loss_function_differentiates_like_the_library():
    torch.manual_seed(3)
    u_f = torch.randn((2, 300, 64), device=dev())
    u_s = (u_f + 0.05 * torch.randn_like(u_f)).requires_grad_(True)
    twin = u_s.detach().clone().requires_grad_(True)
    for reduction, scale in (("mean", 1.0), ("batch", u_f[0].numel())):
        u_s.grad = twin.grad = None
        loss = vd.velocity_distillation_loss(u_s, u_f, reduction)
        (3.0 * loss).backward()
        ref = torch.nn.functional.mse_loss(twin.double(), u_f.double()) * scale
        (3.0 * ref).backward()
        assert loss.dtype == torch.float64 and abs(loss.item() - ref.item()) <= 1e-6 * ref.item()
        torch.testing.assert_close(u_s.grad, twin.grad, rtol=1e-5, atol=1e-12)
    with pytest.raises(ValueError):
        vd.velocity_distillation_loss(u_s.cpu(), u_f.cpu())
