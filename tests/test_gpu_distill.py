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
