"""Pins for the fp64 Adam oracle and its bf16 rounding."""
import math
import numpy as np
import pytest

from oracle import adam_step, bf16_round


def test_first_step_is_sign_update():
    """t = 1, m = v = 0: bias correction gives mhat = g, vhat = g^2, so
    theta' = theta - lr * g / (|g| + eps)."""
    g = np.array([0.5, -2.0, 1e-3, -1e-6])
    th = np.array([1.0, -1.0, 0.25, 3.0])
    lr, eps = 1e-2, 1e-8
    t1, m1, v1, _ = adam_step(th, 0 * th, 0 * th, g, lr, 0.9, 0.999, eps, 0.0, 1, 1.0)
    assert np.allclose(t1, th - lr * g / (np.abs(g) + eps), rtol=1e-14)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)


def test_zero_gradient_zero_state_leaves_theta():
    th = np.array([0.3, -0.7])
    t1, m1, v1, _ = adam_step(th, 0 * th, 0 * th, 0 * th, 1e-3, 0.9, 0.95, 1e-8, 0.0, 5, 1.0)
    assert np.array_equal(t1, th) and not m1.any() and not v1.any()


def test_hand_computed_scalar_example():
    """theta=1, m=0.1, v=0.04, g16=0.5, grad_scale=2 -> g=1; beta=(0.5,0.5), t=2,
    lr=0.1, eps=0, wd=0.1:
      m' = 0.05+0.5 = 0.55 ; v' = 0.02+0.5 = 0.52
      mhat = 0.55/0.75 ; vhat = 0.52/0.75
      theta' = 1 - 0.1*( mhat/sqrt(vhat) + 0.1*1 )"""
    t1, m1, v1, _ = adam_step(1.0, 0.1, 0.04, 0.5, 0.1, 0.5, 0.5, 0.0, 0.1, 2, 2.0)
    mhat = 0.55 / 0.75
    vhat = 0.52 / 0.75
    assert abs(float(m1) - 0.55) < 1e-15 and abs(float(v1) - 0.52) < 1e-15
    assert abs(float(t1) - (1 - 0.1 * (mhat / math.sqrt(vhat) + 0.1))) < 1e-15


def test_constant_gradient_converges_to_unit_steps():
    """Constant g: mhat -> g and vhat -> g^2 exactly at every step (bias correction),
    so each step moves theta by -lr*sign(g) (eps = 0)."""
    th, m, v = np.array([0.0]), np.array([0.0]), np.array([0.0])
    for t in range(1, 30):
        th, m, v, _ = adam_step(th, m, v, np.array([-0.25]), 1e-2, 0.9, 0.99, 0.0, 0.0, t, 1.0)
        assert abs(th[0] - 1e-2 * t) < 1e-12


def test_against_torch_adamw_fp64_many_steps():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    n = 64
    th0 = rng.standard_normal(n)
    p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.01)
    th, m, v = th0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 8):
        g = rng.standard_normal(n)
        p.grad = torch.tensor(g)
        opt.step()
        th, m, v, _ = adam_step(th, m, v, g, 3e-3, 0.9, 0.95, 1e-8, 0.01, t, 1.0)
        assert np.allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_bf16_round_ties_to_even_and_library():
    torch = pytest.importorskip("torch")
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1 and 1 + 2^-7 -> even (1.0)
    assert bf16_round(np.float32(1 + 2 ** -8)) == np.float32(1.0)
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd mantissa) and 1+2^-6 (even) -> 1+2^-6
    assert bf16_round(np.float32(1 + 3 * 2 ** -8)) == np.float32(1 + 2 ** -6)
    assert bf16_round(np.float32(1 + 2 ** -8 + 2 ** -20)) == np.float32(1 + 2 ** -7)
    a = (np.random.default_rng(1).standard_normal(50000) * 10).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    assert np.array_equal(bf16_round(a), ref)
    th, _, _, th16 = adam_step(a[:100], 0 * a[:100], 0 * a[:100], a[100:200], 1e-3, 0.9, 0.95, 1e-8, 0.0, 1, 1.0)
    assert np.array_equal(th16, torch.from_numpy(th.astype(np.float32)).to(torch.bfloat16).float().numpy())
